// Host side of the cnn355 C ABI (include/cnn355.h): architecture grammar, shape inference
// (Sec. 2.2 Eq. 1), connection tables (Sec. 3.1), planning of the per-image step into stages,
// carving of the caller's workspace, and the entry points.  No device memory is allocated here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cctype>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/cnn355.h"
#include "cnn355_dev.h"
#include "cnn355_flowspec.h"

namespace cnn355 {
hipError_t launch_stage(int kind, int n_items, hipStream_t stream, const ProgramDev* d_prog, int s,
                        StatusDev* d_status, const RunArgs& a);
hipError_t launch_stage_pair(int kind_a, int n_a, int kind_b, int n_b, hipStream_t stream, const ProgramDev* d_prog,
                             int s, StatusDev* d_status, const RunArgs& a, bool* done);
hipError_t launch_reset_status(hipStream_t stream, StatusDev* d_status, int clear_label_flag);
hipError_t launch_call_set(hipStream_t stream, CallArgs* d_call, const CallArgs& v);
const void* call_advance_kernel();
const void* stage_kernel(int kind);
const void* stage_pair_kernel(int kind_a, int kind_b);
hipError_t launch_persistent(int grid, bool with_matrix_stages, hipStream_t stream, const ProgramDev* d_prog,
                             StatusDev* d_status, const RunArgs& a);
int persistent_max_blocks_per_cu();
void read_dbg(unsigned long long* out);
hipError_t launch_frontend_batch(hipStream_t stream, const ProgramDev* d_prog, const float* d_images,
                                 long long image_stride, int n_images, int items_per_image, float* d_out);
hipError_t launch_crossing_probe(int G, int stride, hipStream_t stream, tagged_t* buf, int words, int rounds,
                                 unsigned int epoch_base, unsigned int spin_limit, StatusDev* d_status);
hipError_t launch_empty(hipStream_t stream, StatusDev* d_status);
hipError_t launch_resident(int static_id, int grid, size_t lds_bytes, hipStream_t stream, const FlowSpec& spec,
                           const FlowPtrs* d_ptrs, StatusDev* d_status, const RunArgs& a);
int resident_static_id(const FlowSpec& z);
size_t batch_gemm_lds_bytes(const BatchGemm& g);
hipError_t launch_batch_gemm(hipStream_t stream, const BatchGemm& g);
hipError_t launch_batch_pool(hipStream_t stream, const BatchPool& q);
hipError_t launch_batch_outputs(hipStream_t stream, const float* logits, float* probs, long long n_images,
                                int n_classes, int out_units);
hipError_t launch_batch_pack(hipStream_t stream, const BatchPack& q, long long wt_floats);
hipError_t launch_deform(hipStream_t stream, const DeformJob& J);
size_t deform_lds_bytes(const DeformJob& J);
}  // namespace cnn355

using namespace cnn355;

namespace {

constexpr int FE_BATCH = 256;  // images whose front-end outputs are computed ahead of the resident kernel

thread_local std::string g_err;  // message of the last failure that had no handle to carry it

struct ArchLayer {
  int kind = CNN_LAYER_INPUT;
  int maps = 0, h = 0, w = 0, K = 0, S = 0;  // K, S: the y (row) values of kernel / pooling rectangle and skipping factor
  int Kx = 0, Sx = 0;                        // their x (column) values
};

int fail(std::string* where, int code, const std::string& msg) {
  if (where) *where = msg;
  g_err = msg;
  return code;
}

// ---- grammar: <C>x<H>x<W> { -<M>C<K>[S<s>] | -MP<K> | -<N>N }+ ; K, s: <k> or <ky>x<kx> -------------
bool take_number(const std::string& s, size_t& pos, int& v) {
  if (pos >= s.size() || !std::isdigit((unsigned char)s[pos])) return false;
  long long x = 0;
  while (pos < s.size() && std::isdigit((unsigned char)s[pos])) {
    x = x * 10 + (s[pos] - '0');
    if (x > (1 << 20)) return false;
    ++pos;
  }
  v = (int)x;
  return true;
}

// <k> (both directions) or <ky>x<kx> (Sec. 2.2, 2.3: an x and a y value each)
bool take_pair(const std::string& s, size_t& pos, int& vy, int& vx) {
  if (!take_number(s, pos, vy)) return false;
  vx = vy;
  if (pos < s.size() && s[pos] == 'x') {
    ++pos;
    if (!take_number(s, pos, vx)) return false;
  }
  return true;
}

int parse_arch(const char* arch, std::vector<ArchLayer>& out, std::string* err) {
  if (!arch) return fail(err, CNN_E_ARG, "architecture string is NULL");
  const std::string s(arch);
  std::vector<std::string> tok;
  {
    size_t a = 0;
    while (true) {
      size_t b = s.find('-', a);
      tok.push_back(s.substr(a, b == std::string::npos ? std::string::npos : b - a));
      if (b == std::string::npos) break;
      a = b + 1;
    }
  }
  out.clear();
  {
    ArchLayer in;
    size_t p = 0;
    const std::string& t = tok[0];
    if (!take_number(t, p, in.maps) || p >= t.size() || t[p++] != 'x' || !take_number(t, p, in.h) ||
        p >= t.size() || t[p++] != 'x' || !take_number(t, p, in.w) || p != t.size())
      return fail(err, CNN_E_SYNTAX, "input must be <C>x<H>x<W>, got '" + t + "'");
    if (in.maps < 1 || in.h < 1 || in.w < 1) return fail(err, CNN_E_SHAPE, "empty input '" + t + "'");
    out.push_back(in);
  }
  bool fc_seen = false;
  for (size_t ti = 1; ti < tok.size(); ++ti) {
    const std::string& t = tok[ti];
    const ArchLayer prev = out.back();
    ArchLayer l;
    size_t p = 0;
    if (t.size() >= 2 && t[0] == 'M' && t[1] == 'P') {
      p = 2;
      if (!take_pair(t, p, l.K, l.Kx) || p != t.size()) return fail(err, CNN_E_SYNTAX, "bad pooling token '" + t + "'");
      if (prev.kind != CNN_LAYER_CONV)
        return fail(err, CNN_E_SYNTAX, "'" + t + "': max-pooling must follow a convolutional layer");
      if (l.K < 1 || l.Kx < 1) return fail(err, CNN_E_SHAPE, "'" + t + "': empty pooling rectangle");
      if (prev.h % l.K || prev.w % l.Kx)
        return fail(err, CNN_E_SHAPE, "'" + t + "': rectangle does not tile a " + std::to_string(prev.h) + "x" +
                                          std::to_string(prev.w) + " map");
      l.kind = CNN_LAYER_POOL;
      l.maps = prev.maps;
      l.h = prev.h / l.K;
      l.w = prev.w / l.Kx;
    } else {
      int n = 0;
      if (!take_number(t, p, n) || p >= t.size()) return fail(err, CNN_E_SYNTAX, "bad token '" + t + "'");
      const char c = t[p++];
      if (c == 'C') {
        if (!take_pair(t, p, l.K, l.Kx)) return fail(err, CNN_E_SYNTAX, "bad kernel size in '" + t + "'");
        if (p < t.size()) {
          if (t[p++] != 'S' || !take_pair(t, p, l.S, l.Sx) || p != t.size())
            return fail(err, CNN_E_SYNTAX, "bad skipping factor in '" + t + "'");
        }
        if (fc_seen) return fail(err, CNN_E_SYNTAX, "'" + t + "': convolution after a fully connected layer");
        if (n < 1 || l.K < 1 || l.Kx < 1) return fail(err, CNN_E_SHAPE, "'" + t + "': empty layer");
        l.kind = CNN_LAYER_CONV;
        l.maps = n;
        // Eq. 1 of Sec. 2.2, rounded down: the kernel stays completely inside the map
        l.h = prev.h >= l.K ? (prev.h - l.K) / (l.S + 1) + 1 : 0;
        l.w = prev.w >= l.Kx ? (prev.w - l.Kx) / (l.Sx + 1) + 1 : 0;
        if (l.h < 1 || l.w < 1)
          return fail(err, CNN_E_SHAPE, "'" + t + "': kernel larger than its " + std::to_string(prev.h) + "x" +
                                            std::to_string(prev.w) + " input");
      } else if (c == 'N') {
        if (p != t.size()) return fail(err, CNN_E_SYNTAX, "bad token '" + t + "'");
        if (n < 1) return fail(err, CNN_E_SHAPE, "'" + t + "': empty layer");
        l.kind = CNN_LAYER_FC;
        l.maps = n;
        l.h = l.w = 1;
        fc_seen = true;
      } else {
        return fail(err, CNN_E_SYNTAX, "bad token '" + t + "'");
      }
    }
    out.push_back(l);
  }
  if (out.size() < 2 || out.back().kind != CNN_LAYER_FC)
    return fail(err, CNN_E_SYNTAX, "the last layer must be fully connected (<N>N)");
  return CNN_OK;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Does a convolutional layer go to the matrix cores?  Only where the contraction is really dense:
// at least 64 output maps, at least 256 terms per output (input maps x kernel taps), and a map that
// one wavefront set can tile (32-pixel tiles, at most 4 per wavefront).  The table must be full.
bool mfma_shape_ok(int Mi, int K, int Mo, int Ho, int Wo) {
  const long long Kd = (long long)Mi * K * K, P = (long long)Ho * Wo;
  return Mo >= 64 && Kd >= 256 && P >= 16 && P <= MAX_TILE_PIX && (P + 31) / 32 <= (WG / 64) * 4;
}
// The same for the delta pull through such a layer, which is FP's mirror image when the skipping
// factor is 0: rows = input maps, contraction over (output map, tap), columns = input pixels.
bool mfma_bwd_shape_ok(int Mi, int K, int S, int Mo, int Hi, int Wi) {
  const long long Kd = (long long)Mo * K * K, P = (long long)Hi * Wi;
  return S == 0 && Mi >= 32 && Kd >= 256 && P >= 16 && P <= MAX_TILE_PIX && (P + 31) / 32 <= (WG / 64) * 4;
}
// Weight gradients of such a layer as a matrix product over the output pixels: rows = output maps,
// columns = (input map, tap); the deltas of 32 maps over the whole output map must fit in LDS next
// to at least one input map.
bool mfma_wgrad_shape_ok(int Mi, int K, int Mo, int Hi, int Wi, int Ho, int Wo) {
  const long long cols = (long long)Mi * K * K, P = (long long)Ho * Wo;
  // (measured: below some 300 000 weights the vector kernel, which visits the winners only, is as fast)
  return Mo >= 64 && cols >= 256 && Mo * cols >= 300000 && P >= 4 && 32 * (P + 2) + P + (long long)Hi * Wi + 64 <= LDS_FLOATS;
}
int ceil_log2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

// A bump allocator over the caller's workspace; with base == NULL it only measures.
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  template <class T>
  T* take(size_t count) {
    off = align_up(off, 256);
    T* p = base ? (T*)(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

}  // namespace

struct cnn {
  std::vector<ArchLayer> arch;
  std::vector<int> dev_of_arch;  // arch layer -> index in prog.layers (pool -> its conv), -1 for input
  std::vector<std::vector<uint8_t>> tables;  // per convolutional layer, [Mo][Mi]
  // fixed front-end
  int fe_n = 0, fe_K = 0, fe_src_n = 0;
  std::vector<float> fe_filters;
  std::vector<int> fe_src;

  ProgramDev prog;  // host copy with device pointers
  ProgramDev* d_prog = nullptr;
  StatusDev* d_status = nullptr;
  // stage mode: the launches of graph_images images as one graph, replayed (one for training, one forward only)
  CallArgs* d_call = nullptr;
  int graph_images = 0;         // 0: every stage of every image is launched by itself (the default: measured, a
                                //   replayed kernel node costs what a launch costs once the kernels do real work)
  hipGraphExec_t graph_exec[2] = {nullptr, nullptr};
  int graph_built_for[2] = {0, 0};
  float* d_weights = nullptr;
  float* d_grad = nullptr;
  float* d_fe_filters = nullptr;
  int* d_fe_src = nullptr;
  float* d_fe_out = nullptr;
  float* d_fe_batch = nullptr;  // resident mode: front-end outputs of FE_BATCH images at a time
  float* d_mm_part = nullptr;   // partial sums of the matrix-core forward pass (one layer at a time)
  int use_mfma = 1;
  int out_units = CNN_OUTPUT_SOFTMAX_XENT;
  struct ConvBuf {
    float *act, *out, *delta, *dact;
    uint8_t* arg;
    int *argyx, *csr_ptr, *csr_idx, *csc_ptr, *csc_j, *csc_slot;
  };
  struct FcBuf { float *act, *delta, *dact; };
  std::vector<ConvBuf> conv_buf;
  std::vector<FcBuf> fc_buf;
  struct HostTable { std::vector<int> csr_ptr, csr_idx, csc_ptr, csc_j, csc_slot; int max_conn = 0, max_back = 0; };
  std::vector<HostTable> host_tables;  // per convolutional layer, rebuilt by plan()

  // resident mode
  FlowSpec flow;                // the plan (plain integers); the resident kernel takes it by value
  FlowPtrs flow_ptrs;           // where the layers and the exchange buffers lie on the device
  FlowPtrs* d_flow_ptrs = nullptr;
  int flow_static_id = 0;       // > 0: the plan equals that of a kernel compiled for a fixed network
  // a resident kernel compiled for this handle's own network and loaded from a code object
  hipModule_t special_module = nullptr;
  hipFunction_t special_func = nullptr;
  FlowSpec special_plan;        // the plan that code object was compiled for
  bool special_active = false;  // the current plan equals it: calls go to special_func
  tagged_t* d_xbuf = nullptr;   // every exchange buffer, one after the other
  size_t xbuf_words = 0;
  bool flow_ok = false;
  std::string flow_why;         // why resident mode cannot run this network
  int team_ranks = 0, team_stride = 0;  // 0 = automatic
  unsigned long long epoch = 0; // images run in resident mode so far (their tags)

  size_t n_weights = 0, n_weights_max = 0;
  size_t image_size = 0;
  int n_classes = 0;
  hipStream_t stream = nullptr;
  int device = 0;               // the device that was current at cnn_create
  int mode = CNN_MODE_STAGES;
  int n_cu = 0, grid_override = 0, coop_ok = 0, max_blocks_per_cu = 1;
  unsigned int spin_limit = 1u << 22;
  int barrier_kind = 1;
  bool need_status_reset = true;
  std::string err;
};

namespace {

int hip_fail(cnn* net, hipError_t e, const char* what) {
  return fail(net ? &net->err : nullptr, CNN_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(net, call)                                   \
  do {                                                       \
    hipError_t e_ = (call);                                  \
    if (e_ != hipSuccess) return hip_fail(net, e_, #call);   \
  } while (0)

// Lay the workspace out.  With net->d_* pointers filled when base != NULL.
size_t carve(cnn* net, void* base) {
  Carver c(base);
  const auto& A = net->arch;
  // upper bound on weights: every table full
  size_t nw = 0;
  for (size_t l = 1; l < A.size(); ++l) {
    if (A[l].kind == CNN_LAYER_CONV) nw += (size_t)A[l].maps * (1 + (size_t)A[l - 1].maps * A[l].K * A[l].Kx);
    if (A[l].kind == CNN_LAYER_FC) nw += (size_t)A[l].maps * (1 + (size_t)A[l - 1].maps * A[l - 1].h * A[l - 1].w);
  }
  net->n_weights_max = nw;
  net->d_prog = c.take<ProgramDev>(1);
  net->d_status = c.take<StatusDev>(1);
  net->d_call = c.take<CallArgs>(1);
  net->d_weights = c.take<float>(nw);
  net->d_grad = c.take<float>(nw);
  net->d_fe_filters = c.take<float>((size_t)A[0].maps * MAX_FRONTEND_K * MAX_FRONTEND_K);
  net->d_fe_src = c.take<int>(A[0].maps);
  net->d_fe_out = c.take<float>((size_t)A[0].maps * A[0].h * A[0].w);
  net->d_fe_batch = c.take<float>((size_t)FE_BATCH * A[0].maps * A[0].h * A[0].w);
  {
    size_t mm = 0;
    for (size_t l = 1; l < A.size(); ++l)
      if (A[l].kind == CNN_LAYER_CONV) {
        if (mfma_shape_ok(A[l - 1].maps, A[l].K, A[l].maps, A[l].h, A[l].w))
          mm = std::max(mm, (size_t)MFMA_MAX_SLICES * A[l].maps * A[l].h * A[l].w);
        if (l >= 2 && mfma_bwd_shape_ok(A[l - 1].maps, A[l].K, A[l].S, A[l].maps, A[l - 1].h, A[l - 1].w))
          mm = std::max(mm, (size_t)MFMA_MAX_SLICES * A[l - 1].maps * A[l - 1].h * A[l - 1].w);
      }
    net->d_mm_part = c.take<float>(mm);
  }
  net->d_flow_ptrs = c.take<FlowPtrs>(1);
  {  // resident mode: tagged exchange buffers, sized for any team (see plan_flow for the split)
    size_t words = 0, last_maps = 0, first_fc = 0, n_fc_seen = 0;
    for (size_t l = 1; l < A.size(); ++l) {
      if (A[l].kind == CNN_LAYER_CONV) {
        const bool pooled = l + 1 < A.size() && A[l + 1].kind == CNN_LAYER_POOL;
        const size_t small = pooled ? (size_t)A[l + 1].maps * A[l + 1].h * A[l + 1].w : (size_t)A[l].maps * A[l].h * A[l].w;
        words += 3 * 2 * small;  // pooled outputs, deltas, winner coordinates; two images in flight
        words += 2 * 256 * (small / A[l].maps);  // pulled sums of the shares of a map's pull (fewer than 256 of them)
        words += 2 * (size_t)A[l].maps * A[l - 1].maps * (A[l].K * A[l].Kx + 4);  // adjusted filters on their way to the forward copies
        last_maps = A[l].maps;
      } else if (A[l].kind == CNN_LAYER_FC) {
        if (!first_fc) first_fc = A[l].maps;
        // a second fully connected layer held by columns: partial sums of up to 256 ranks, deltas of its inputs
        if (++n_fc_seen == 2) words += 2 * (size_t)256 * A[l].maps + 2 * (size_t)A[l - 1].maps * A[l - 1].h * A[l - 1].w;
      }
    }
    words += 2 * std::min<size_t>(last_maps, 256) * first_fc + 2 * first_fc;
    net->xbuf_words = words;
    net->d_xbuf = c.take<tagged_t>(words);
  }
  net->conv_buf.clear();
  net->fc_buf.clear();
  for (size_t l = 1; l < A.size(); ++l) {
    if (A[l].kind == CNN_LAYER_CONV) {
      // a pooling rectangle of one pixel is the identity: the pooled values are the activations
      const bool pooled = l + 1 < A.size() && A[l + 1].kind == CNN_LAYER_POOL && (A[l + 1].K > 1 || A[l + 1].Kx > 1);
      const size_t full = (size_t)A[l].maps * A[l].h * A[l].w;
      const size_t small = pooled ? (size_t)A[l + 1].maps * A[l + 1].h * A[l + 1].w : full;
      const size_t nc = (size_t)A[l].maps * A[l - 1].maps;
      cnn::ConvBuf b;
      b.act = c.take<float>(full);
      b.out = pooled ? c.take<float>(small) : b.act;
      b.delta = c.take<float>(small);
      b.dact = c.take<float>(small);
      b.arg = c.take<uint8_t>(small);
      b.argyx = c.take<int>(small);
      b.csr_ptr = c.take<int>(A[l].maps + 1);
      b.csr_idx = c.take<int>(nc);
      b.csc_ptr = c.take<int>(A[l - 1].maps + 1);
      b.csc_j = c.take<int>(nc);
      b.csc_slot = c.take<int>(nc);
      net->conv_buf.push_back(b);
    } else if (A[l].kind == CNN_LAYER_FC) {
      cnn::FcBuf b;
      b.act = c.take<float>(A[l].maps);
      b.delta = c.take<float>(A[l].maps);
      b.dact = c.take<float>(A[l].maps);
      net->fc_buf.push_back(b);
    }
  }
  return align_up(c.off, 256);
}

// Choose the band of conv rows one workgroup computes in the forward stage.
int plan_conv_fwd(const LayerDev& L, Stage& st, int n_cu, std::string* err) {
  const int Kp = L.Kp, Wo = L.Wo, Ho = L.Ho;
  const int target = 256;
  int rows = 0;
  if (Kp * Wo <= WG) {
    // the largest band of at most 256 pixels that still gives `want` work items; if no band does,
    // the smallest band (most items) of at least one wavefront of pixels
    const int want = 128;
    int max_rows = std::min(Ho, (WG / Wo) / Kp * Kp);
    for (int r = max_rows; r >= Kp; r -= Kp)
      if ((long long)L.Mo * ((Ho + r - 1) / r) >= want) { rows = r; break; }
    if (!rows) {
      rows = Kp;
      while (rows * Wo < 64 && rows + Kp <= max_rows) rows += Kp;
    }
    st.pix_per_thread = 1;
  } else {
    if (Kp * Wo > MAX_TILE_PIX) return fail(err, CNN_E_SHAPE, "convolutional map too wide for the forward kernel");
    rows = std::min(Ho, (MAX_TILE_PIX / Wo) / Kp * Kp);
    while (rows > Kp && (long long)L.Mo * ((Ho + rows - 1) / rows) < target) rows -= Kp;
    st.pix_per_thread = 2;
  }
  st.tile_rows = rows;
  st.n_tiles = (Ho + rows - 1) / rows;
  st.n_items = L.Mo * st.n_tiles;
  const int map_sz = ((rows - 1) * (L.S + 1) + L.K) * L.Wi;
  const int chunk = std::min({LDS_IN / map_sz, LDS_AUX / (L.K * L.Kx), L.max_conn});
  if (chunk < 1) return fail(err, CNN_E_SHAPE, "convolution input rows do not fit the LDS staging area");
  st.chunk = chunk;
  st.tw_log2 = ceil_log2(std::min(map_sz, WG));
  // A few items more than compute units would leave most units idle through a second round: then two (or
  // three) output maps per item, which share the staged input maps (full table, all of them in one chunk).
  st.rows_per_wg = 1;
  if (L.full_table && L.Mi <= chunk && st.n_items > n_cu && st.n_items <= 3 * n_cu && st.n_items % n_cu < n_cu / 2 && st.n_items % n_cu != 0) {
    const int mp = (st.n_items + n_cu - 1) / n_cu;
    st.rows_per_wg = mp;
    st.n_items = ((L.Mo + mp - 1) / mp) * st.n_tiles;
  }
  return CNN_OK;
}

// Forward (CSR), backward (CSC) and slot tables of one convolutional layer from its 0/1 table.
void build_tables(int Mo, int Mi, const std::vector<uint8_t>& table, cnn::HostTable& T) {
  T = cnn::HostTable();
  T.csr_ptr.assign(Mo + 1, 0);
  T.csc_ptr.assign(Mi + 1, 0);
  for (int j = 0; j < Mo; ++j) {
    for (int i = 0; i < Mi; ++i)
      if (table[(size_t)j * Mi + i]) T.csr_idx.push_back(i);
    T.csr_ptr[j + 1] = (int)T.csr_idx.size();
    T.max_conn = std::max(T.max_conn, T.csr_ptr[j + 1] - T.csr_ptr[j]);
  }
  for (int i = 0; i < Mi; ++i) {
    for (int j = 0; j < Mo; ++j)
      for (int s = T.csr_ptr[j]; s < T.csr_ptr[j + 1]; ++s)
        if (T.csr_idx[s] == i) { T.csc_j.push_back(j); T.csc_slot.push_back(s); }
    T.csc_ptr[i + 1] = (int)T.csc_j.size();
    T.max_back = std::max(T.max_back, T.csc_ptr[i + 1] - T.csc_ptr[i]);
  }
}

// Every size a kernel relies on, re-derived from the finished plan: a stage whose operands do
// not fit its LDS areas or its thread mapping is refused here, never launched.
int check_plan(cnn* net) {
  const ProgramDev& P = net->prog;
  auto bad = [&](int s, const char* what) {
    return fail(&net->err, CNN_E_SHAPE, "stage " + std::to_string(s) + ": " + what);
  };
  for (int s = 0; s < P.n_stages; ++s) {
    const Stage& st = P.stages[s];
    const LayerDev& L = P.layers[st.layer];
    if (st.n_items < 1) return bad(s, "no work items");
    switch (st.kind) {
      case ST_CONV_FWD: {
        const int P_max = st.tile_rows * L.Wo;
        const int map_sz = ((st.tile_rows - 1) * (L.S + 1) + L.K) * L.Wi;
        if (st.tile_rows < L.Kp || st.tile_rows % L.Kp) return bad(s, "row band not a multiple of the pooling size");
        if (st.pix_per_thread == 1 ? P_max > WG : P_max > MAX_TILE_PIX) return bad(s, "row band too large");
        if (st.pix_per_thread != 1 && st.pix_per_thread != 2) return bad(s, "bad pixels per thread");
        if (st.chunk < 1 || (long long)st.chunk * map_sz > LDS_IN) return bad(s, "input chunk exceeds the LDS input area");
        if (st.chunk * L.K * L.Kx > LDS_AUX) return bad(s, "filter chunk exceeds the LDS filter area");
        if (st.rows_per_wg < 1 || st.n_tiles * st.tile_rows < L.Ho || st.n_items != ((L.Mo + st.rows_per_wg - 1) / st.rows_per_wg) * st.n_tiles)
          return bad(s, "row bands do not cover the maps");
        if (st.rows_per_wg > 1 && (!L.full_table || L.Mi > st.chunk)) return bad(s, "output maps of one work item must share one chunk of input maps");
        if ((1 << st.tw_log2) > WG) return bad(s, "staging width");
        break;
      }
      case ST_CONV_BWD: {
        const int pt = 1 << st.tw_log2;
        if (st.chunk < 1 || (long long)st.chunk * (L.Ho + 1) * (L.Wo + 1) > LDS_IN) return bad(s, "delta chunk exceeds its LDS area");
        if (st.chunk * L.K * L.Kx > LDS_AUX) return bad(s, "filter chunk exceeds its LDS area");
        if (pt < 1 || pt > WG || st.n_tiles * pt < L.Hi * L.Wi || st.n_items != L.Mi * st.n_tiles) return bad(s, "pixel tiles do not cover the map");
        if (st.layer < 1) return bad(s, "no layer below");
        break;
      }
      case ST_CONV_WGRAD: {
        if (st.chunk < 1 || (long long)st.chunk * L.Hi * L.Wi > LDS_IN) return bad(s, "input maps exceed the LDS input area");
        if (L.Hp * L.Wp > LDS_AUX || L.Hp * L.Wp > LDS_AUX2) return bad(s, "pooled map exceeds its LDS area");
        if (st.n_tiles * st.chunk < L.max_conn || st.n_items != L.Mo * st.n_tiles) return bad(s, "chunks do not cover the connections");
        if ((1 << st.tw_log2) > WG) return bad(s, "staging width");
        break;
      }
      case ST_FC_FWD:
        if (st.rows_per_wg < 1 || st.rows_per_wg > WG / 64 || (st.rows_per_wg & (st.rows_per_wg - 1))) return bad(s, "rows per workgroup");
        if (st.n_items * st.rows_per_wg < L.n_out) return bad(s, "rows not covered");
        break;
      case ST_HEAD:
        if (L.n_out > LDS_AUX || L.n_out > LDS_AUX2 || st.n_items != 1) return bad(s, "output layer too wide");
        break;
      case ST_FC_BWD:
        if (L.n_out > LDS_AUX) return bad(s, "layer too wide");
        if (st.cm_log2 < 0 || st.cm_log2 > 8 || (st.n_items << st.cm_log2) < L.n_in) return bad(s, "columns not covered");
        break;
      case ST_FRONTEND:
        if (st.n_items * WG < P.fe.n_filters * P.fe.H * P.fe.W) return bad(s, "pixels not covered");
        break;
      case ST_CONV_FWD_MFMA: {
        const int KK = L.K * L.K, HiWi = L.Hi * L.Wi, Pn = L.Ho * L.Wo;
        const int NT = (Pn + 31) / 32, waves = WG / 64, KW = NT >= waves ? 1 : waves / NT;
        const int WP = st.chunk * KK + 1 + ((st.chunk * KK) & 1);
        if (L.rect || !L.full_table || !mfma_shape_ok(L.Mi, L.K, L.Mo, L.Ho, L.Wo)) return bad(s, "layer not fit for the matrix-core kernel");
        if (st.chunk < 1 || (long long)st.chunk * HiWi + 32LL * WP + (long long)st.chunk * KK > LDS_FLOATS) return bad(s, "chunk exceeds LDS");
        if (st.n_tiles < 1 || st.n_tiles > L.Mi || st.n_items != ((L.Mo + 31) / 32) * st.n_tiles) return bad(s, "slices do not cover the input maps");
        if (st.rows_per_wg != st.n_tiles || st.rows_per_wg > MFMA_MAX_SLICES) return bad(s, "too many partial-sum planes");
        if (KW > 1 && (long long)KW * NT * 1024 > LDS_FLOATS) return bad(s, "k splits do not fit LDS");
        if (((L.Mi + st.n_tiles - 1) / st.n_tiles) * (st.n_tiles - 1) >= L.Mi) return bad(s, "an empty slice");
        break;
      }
      case ST_CONV_BWD_MFMA: {
        const int KK = L.K * L.K, HWd = (L.Hi + L.K - 1) * (L.Wi + L.K - 1), Pn = L.Hi * L.Wi;
        const int NT = (Pn + 31) / 32, waves = WG / 64, KW = NT >= waves ? 1 : waves / NT;
        const int WP = st.chunk * KK + 1 + ((st.chunk * KK) & 1);
        if (net->mode != CNN_MODE_STAGES) return bad(s, "the matrix-core pull is planned for the stage-launch mode only");
        if (L.rect || !L.full_table || !mfma_bwd_shape_ok(L.Mi, L.K, L.S, L.Mo, L.Hi, L.Wi)) return bad(s, "layer not fit for the matrix-core pull");
        if (st.chunk < 1 || (long long)st.chunk * HWd + 32LL * WP + (long long)st.chunk * KK > LDS_FLOATS) return bad(s, "chunk exceeds LDS");
        if (st.n_tiles < 1 || st.n_tiles > L.Mo || st.n_items != ((L.Mi + 31) / 32) * st.n_tiles) return bad(s, "slices do not cover the output maps");
        if (st.rows_per_wg != st.n_tiles || st.rows_per_wg > MFMA_MAX_SLICES) return bad(s, "too many partial-sum planes");
        if (KW > 1 && (long long)KW * NT * 1024 > LDS_FLOATS) return bad(s, "k splits do not fit LDS");
        if (((L.Mo + st.n_tiles - 1) / st.n_tiles) * (st.n_tiles - 1) >= L.Mo) return bad(s, "an empty slice");
        if (st.layer < 1 || P.layers[st.layer - 1].kind != L_CONV) return bad(s, "no convolutional layer below");
        break;
      }
      case ST_CONV_WGRAD_MFMA: {
        const int KK = L.K * L.K, Pn = L.Ho * L.Wo, WP = Pn + 1 + (Pn & 1);
        const int NT = (std::min(st.chunk, L.Mi) * KK + 31) / 32, waves = WG / 64, KW = NT >= waves ? 1 : waves / NT;
        if (net->mode != CNN_MODE_STAGES) return bad(s, "the matrix-core gradient is planned for the stage-launch mode only");
        if (L.rect || !L.full_table || !mfma_wgrad_shape_ok(L.Mi, L.K, L.Mo, L.Hi, L.Wi, L.Ho, L.Wo)) return bad(s, "layer not fit for the matrix-core gradient");
        if (st.chunk < 1 || (long long)st.chunk * L.Hi * L.Wi + 32LL * WP + Pn > LDS_FLOATS) return bad(s, "chunk exceeds LDS");
        if (NT > 4 * waves) return bad(s, "too many column tiles");
        if (KW * NT * 1024 > LDS_FLOATS) return bad(s, "k splits do not fit LDS");
        if (st.n_tiles * st.chunk < L.Mi || (st.n_tiles - 1) * st.chunk >= L.Mi || st.n_items != ((L.Mo + 31) / 32) * st.n_tiles) return bad(s, "chunks do not cover the input maps");
        break;
      }
      case ST_CONV_BWD_EPI:
        if (st.rows_per_wg < 1 || st.rows_per_wg > MFMA_MAX_SLICES) return bad(s, "partial-sum planes");
        if (st.chunk < 1 || st.n_items != (L.Mi + st.chunk - 1) / st.chunk) return bad(s, "work items do not cover the input maps");
        if (st.layer < 1) return bad(s, "no layer below");
        break;
      case ST_CONV_EPI:
        if (st.rows_per_wg < 1 || st.rows_per_wg > MFMA_MAX_SLICES) return bad(s, "partial-sum planes");
        if (st.chunk < 1 || st.n_items != (L.Mo + st.chunk - 1) / st.chunk) return bad(s, "work items do not cover the maps");
        if (L.Ho * L.Wo > MAX_TILE_PIX) return bad(s, "map too large");
        if (st.chunk > 1 && st.chunk * L.Ho * L.Wo > WG) return bad(s, "maps of a work item exceed its lanes");
        break;
      default:
        return bad(s, "unknown stage kind");
    }
  }
  return CNN_OK;
}

void plan_flow(cnn* net);
void drop_stage_graphs(cnn* net);

// Build layer descriptors, tables and the stage list on the host (no device call).  Works on
// a handle whose workspace pointers are NULL (measuring / checking only).
int plan(cnn* net) {
  drop_stage_graphs(net);   // (their nodes carry the stage list that is about to change)
  const auto& A = net->arch;
  ProgramDev& P = net->prog;
  std::memset(&P, 0, sizeof(P));
  net->dev_of_arch.assign(A.size(), -1);
  net->host_tables.assign(net->tables.size(), cnn::HostTable());
  int nl = 0, conv_i = 0, fc_i = 0;
  std::vector<int> conv_of_dev(MAX_LAYERS, -1);  // descriptor index -> convolutional layer index
  size_t woff = 0;
  const float* below = nullptr;  // output buffer of the layer below
  const bool fe = net->fe_n > 0;
  bool has_below = fe;           // (pointers are all NULL when only measuring)
  if (fe) below = net->d_fe_out;
  for (size_t l = 1; l < A.size(); ++l) {
    if (A[l].kind == CNN_LAYER_POOL) { net->dev_of_arch[l] = nl - 1; continue; }
    if (nl >= MAX_LAYERS) return fail(&net->err, CNN_E_SHAPE, "too many layers");
    LayerDev& L = P.layers[nl];
    L.in_is_image = !has_below;
    L.in = below;
    if (A[l].kind == CNN_LAYER_CONV) {
      const bool pooled = l + 1 < A.size() && A[l + 1].kind == CNN_LAYER_POOL;
      L.kind = L_CONV;
      L.Mi = A[l - 1].maps; L.Hi = A[l - 1].h; L.Wi = A[l - 1].w;
      L.Mo = A[l].maps; L.Ho = A[l].h; L.Wo = A[l].w;
      L.K = A[l].K; L.S = A[l].S; L.Kx = A[l].Kx; L.Sx = A[l].Sx;
      L.Kp = pooled ? A[l + 1].K : 1;
      L.Kpx = pooled ? A[l + 1].Kx : 1;
      L.rect = (L.K != L.Kx || L.S != L.Sx || L.Kp != L.Kpx) ? 1 : 0;
      L.Hp = L.Ho / L.Kp; L.Wp = L.Wo / L.Kpx;
      if (L.Ho >= 65536 || L.Wo >= 65536) return fail(&net->err, CNN_E_SHAPE, "map too large");
      if (L.Hp * L.Wp > MAX_POOLED_PIX)
        return fail(&net->err, CNN_E_SHAPE, "pooled map has more than " + std::to_string(MAX_POOLED_PIX) + " positions");
      if (L.Hi * L.Wi > LDS_IN || (L.Ho + 1) * (L.Wo + 1) > LDS_IN)
        return fail(&net->err, CNN_E_SHAPE, "a map has more than " + std::to_string(LDS_IN) + " pixels");
      if (L.Kp > 15 || L.Kpx > 15) return fail(&net->err, CNN_E_SHAPE, "pooling rectangle larger than 15x15");
      const cnn::ConvBuf& b = net->conv_buf[conv_i];
      L.act = b.act; L.out = b.out; L.delta = b.delta; L.dact = b.dact; L.arg = b.arg; L.argyx = b.argyx;
      L.csr_ptr = b.csr_ptr; L.csr_idx = b.csr_idx; L.csc_ptr = b.csc_ptr; L.csc_j = b.csc_j; L.csc_slot = b.csc_slot;
      L.mm_part = net->d_mm_part;
      conv_of_dev[nl] = conv_i;
      build_tables(L.Mo, L.Mi, net->tables[conv_i], net->host_tables[conv_i]);
      L.max_conn = net->host_tables[conv_i].max_conn;
      L.full_table = net->host_tables[conv_i].csr_idx.size() == (size_t)L.Mo * L.Mi;
      const size_t n_conn = net->host_tables[conv_i].csr_idx.size();
      L.b_canon = (long long)woff;
      L.w_canon = (long long)(woff + L.Mo);
      woff += L.Mo + n_conn * L.K * L.Kx;
      ++conv_i;
    } else {
      L.kind = L_FC;
      L.n_in = A[l - 1].maps * A[l - 1].h * A[l - 1].w;
      L.n_out = A[l].maps;
      L.is_output = (l + 1 == A.size());
      L.out_units = L.is_output ? net->out_units : 0;
      if (L.n_out > MAX_FC_OUT)
        return fail(&net->err, CNN_E_SHAPE, "fully connected layer wider than " + std::to_string(MAX_FC_OUT));
      const cnn::FcBuf& b = net->fc_buf[fc_i];
      L.act = b.act; L.out = b.act; L.delta = b.delta; L.dact = b.dact;
      L.b_canon = (long long)woff;
      L.w_canon = (long long)(woff + L.n_out);
      woff += (size_t)L.n_out * (1 + (size_t)L.n_in);
      ++fc_i;
    }
    // (a handle that only plans, without a workspace, has no weights to point into)
    L.bias = net->d_weights ? net->d_weights + L.b_canon : nullptr;
    L.w = net->d_weights ? net->d_weights + L.w_canon : nullptr;
    below = L.out;
    has_below = true;
    net->dev_of_arch[l] = nl;
    ++nl;
  }
  P.n_layers = nl;
  P.n_classes = A.back().maps;
  net->n_classes = P.n_classes;
  net->n_weights = woff;
  P.has_frontend = fe ? 1 : 0;
  if (fe) {
    FrontendDev& F = P.fe;
    F.n_filters = net->fe_n; F.K = net->fe_K; F.n_src = net->fe_src_n;
    F.H = A[0].h; F.W = A[0].w;
    F.Hr = F.H + F.K - 1; F.Wr = F.W + F.K - 1;
    F.filters = net->d_fe_filters; F.src = net->d_fe_src; F.out = net->d_fe_out;
    net->image_size = (size_t)F.n_src * F.Hr * F.Wr;
  } else {
    net->image_size = (size_t)A[0].maps * A[0].h * A[0].w;
  }

  // ---- stage list ------------------------------------------------------------------------
  int ns = 0;
  auto add = [&](int kind, int layer, int n_items, int barrier, int train_only) -> Stage& {
    Stage& s = P.stages[ns++];
    s.kind = kind; s.layer = layer; s.n_items = n_items; s.barrier_after = barrier; s.train_only = train_only;
    return s;
  };
  if (4 * nl + 4 > MAX_STAGES) return fail(&net->err, CNN_E_SHAPE, "too many stages");
  if (fe) add(ST_FRONTEND, 0, (net->fe_n * A[0].h * A[0].w + WG - 1) / WG, 1, 0);
  for (int l = 0; l < nl; ++l) {  // forward, bottom up
    LayerDev& L = P.layers[l];
    if (L.kind == L_CONV && net->use_mfma && !L.rect && L.full_table && mfma_shape_ok(L.Mi, L.K, L.Mo, L.Ho, L.Wo)) {
      // wide layer: implicit GEMM on the matrix cores, the contraction split over workgroups, then
      // a second stage that adds the partial sums and does what follows the sum
      const int n_cu = net->n_cu > 0 ? net->n_cu : 256;
      const int KK = L.K * L.K, HiWi = L.Hi * L.Wi, P = L.Ho * L.Wo;
      const int NT = (P + 31) / 32, waves = WG / 64;
      const int KW = NT >= waves ? 1 : waves / NT;
      const int RT = (L.Mo + 31) / 32;
      (void)KW;  // the k splits inside a workgroup are added there: one plane of partial sums per work item
      int KS = std::max(1, std::min({n_cu / RT, L.Mi, MFMA_MAX_SLICES}));
      const int per = (L.Mi + KS - 1) / KS;
      KS = (L.Mi + per - 1) / per;
      const int IC = std::min(per, (LDS_FLOATS - 64) / (HiWi + 33 * KK + 2));
      if (IC < 1) return fail(&net->err, CNN_E_SHAPE, "an input map does not fit the LDS staging area of the matrix-core kernel");
      Stage& s = add(ST_CONV_FWD_MFMA, l, RT * KS, 1, 0);
      s.n_tiles = KS; s.chunk = IC; s.rows_per_wg = KS;
      // maps per work item of the second stage, side by side in its lanes: as many as leave every map its
      // lane groups (one per 8 planes, at most 4), and at least what brings the items down to one round of
      // the compute units where the lanes allow
      const int g_want = std::min((KS + 7) / 8, 4);
      const int mp_keep = std::max(1, WG / (P * g_want)), mp_need = (L.Mo + n_cu - 1) / n_cu;
      const int mp = P >= WG ? 1 : std::max(1, std::min({std::max(mp_keep, std::min(mp_need, WG / P)), L.Mo, 64}));
      Stage& e = add(ST_CONV_EPI, l, (L.Mo + mp - 1) / mp, 1, 0);
      e.rows_per_wg = KS;
      e.chunk = mp;
    } else if (L.kind == L_CONV) {
      Stage& s = add(ST_CONV_FWD, l, 0, 1, 0);
      int rc = plan_conv_fwd(L, s, net->n_cu > 0 ? net->n_cu : 256, &net->err);
      if (rc) return rc;
    } else if (!L.is_output) {
      Stage& s = add(ST_FC_FWD, l, 0, 1, 0);
      // lanes per neuron: about a quarter of its inputs (a few loads per lane), 64 .. 1024
      int lanes = 64;
      while (lanes < WG && lanes * 4 < L.n_in) lanes *= 2;
      s.rows_per_wg = WG / lanes;
      s.n_items = (L.n_out + s.rows_per_wg - 1) / s.rows_per_wg;
    } else {
      add(ST_HEAD, l, 1, 1, 0);
    }
  }
  // backward, top down.  The weights of a convolutional layer are adjusted one stage after the
  // deltas have been pulled through them; that adjustment shares a stage with the next pull.
  int pending_wgrad = -1;
  auto add_wgrad = [&](int l, int barrier) {
    LayerDev& L = P.layers[l];
    if (net->use_mfma && net->mode == CNN_MODE_STAGES && !L.rect && L.full_table &&
        mfma_wgrad_shape_ok(L.Mi, L.K, L.Mo, L.Hi, L.Wi, L.Ho, L.Wo)) {
      // wide layer, one launch per stage: the gradients as a matrix product over the output pixels.
      // Input maps per work item: about one work item per compute unit, whole column tiles of 32
      // where the kernel size allows, at most 64 column tiles, and what LDS holds.
      const int n_cu = net->n_cu > 0 ? net->n_cu : 256;
      const int KK = L.K * L.K, HiWi = L.Hi * L.Wi, Pn = L.Ho * L.Wo;
      const int RT = (L.Mo + 31) / 32;
      const int WP = Pn + 1 + (Pn & 1);
      const int ic_lds = (LDS_FLOATS - 64 - 32 * WP - Pn) / HiWi;
      int unit = 1;
      while ((unit * KK) % 32 != 0 && unit < 8) unit *= 2;   // a few maps that fill whole column tiles, if there are such
      if ((unit * KK) % 32 != 0) unit = 1;
      int ic = (L.Mi + std::max(1, n_cu / RT) - 1) / std::max(1, n_cu / RT);
      ic = (ic + unit - 1) / unit * unit;
      ic = std::max(1, std::min({ic, ic_lds, 64 * 32 / KK, L.Mi}));
      Stage& s = add(ST_CONV_WGRAD_MFMA, l, 0, barrier, 1);
      s.chunk = ic;
      s.n_tiles = (L.Mi + ic - 1) / ic;
      s.n_items = RT * s.n_tiles;
      return;
    }
    Stage& s = add(ST_CONV_WGRAD, l, 0, barrier, 1);
    const int chunk_max = std::min(LDS_IN / (L.Hi * L.Wi), L.max_conn);
    // as many work items as fit one round on the compute units: the connection lists cut into
    // floor(CUs / maps) chunks
    const int n_cu_w = net->n_cu > 0 ? net->n_cu : 256;
    const int want_chunks = std::max(1, n_cu_w / L.Mo);
    int chunk = std::max(1, std::min(chunk_max, (L.max_conn + want_chunks - 1) / want_chunks));
    s.chunk = chunk;
    s.n_tiles = (L.max_conn + chunk - 1) / chunk;
    s.n_items = L.Mo * s.n_tiles;
    s.tw_log2 = ceil_log2(std::min(L.Hi * L.Wi, WG));
  };
  for (int l = nl - 2; l >= 0; --l) {  // layer nl-1 is the output layer, handled by ST_HEAD
    LayerDev& L = P.layers[l];
    if (L.kind == L_FC) {
      Stage& s = add(ST_FC_BWD, l, 0, 1, 1);
      // columns per work item: whole 256-byte (or 128-byte) pieces of a row of W where that still gives most
      // compute units an item, else 64-byte pieces
      s.cm_log2 = (L.n_in / 64 >= 160) ? 6 : (L.n_in / 32 >= 160) ? 5 : 4;
      s.n_items = (L.n_in + (1 << s.cm_log2) - 1) >> s.cm_log2;
    } else {
      if (!L.in_is_image && l > 0) {
        // pull deltas into layer l-1 (reads the old weights of layer l) ...
        const bool with_pending = pending_wgrad >= 0;
        if (with_pending) { add_wgrad(pending_wgrad, 0); pending_wgrad = -1; }
        if (net->use_mfma && net->mode == CNN_MODE_STAGES && !L.rect && L.full_table &&
            mfma_bwd_shape_ok(L.Mi, L.K, L.S, L.Mo, L.Hi, L.Wi)) {
          // wide layer, one launch per stage (the persistent kernel does not hold this stage kind:
          // its registers would slow every other stage): the pull as FP's mirror image on the matrix cores, the contraction over the
          // output maps split over workgroups; the second stage adds the partial sums -- the
          // adjustment of this layer's weights, which the first stage has read, shares its interval
          const int n_cu = net->n_cu > 0 ? net->n_cu : 256;
          const int KK = L.K * L.K, HWd = (L.Hi + L.K - 1) * (L.Wi + L.K - 1);
          const int RT = (L.Mi + 31) / 32;
          int KS = std::max(1, std::min({n_cu / RT, L.Mo, MFMA_MAX_SLICES}));
          const int per = (L.Mo + KS - 1) / KS;
          KS = (L.Mo + per - 1) / per;
          const int IC = std::min(per, (LDS_FLOATS - 64) / (HWd + 33 * KK + 2));
          if (IC >= 1) {
            Stage& s = add(ST_CONV_BWD_MFMA, l, RT * KS, 1, 1);
            s.n_tiles = KS; s.chunk = IC; s.rows_per_wg = KS;
            add_wgrad(l, 0);
            // input maps per work item of the second stage: up to two passes of the lanes over their pixels, but at
            // least 16 items (the weight adjustment that shares the interval leaves few compute units idle)
            const int Pin2 = L.Hi * L.Wi;
            const int mpb = std::max(1, std::min({2 * WG / Pin2, (L.Mi + 15) / 16, L.Mi}));
            Stage& e = add(ST_CONV_BWD_EPI, l, (L.Mi + mpb - 1) / mpb, 1, 1);
            e.rows_per_wg = KS;
            e.chunk = mpb;
            continue;
          }
        }
        Stage& s = add(ST_CONV_BWD, l, 0, 1, 1);
        const int Pin = L.Hi * L.Wi, HW = L.Hp * L.Wp, KK = L.K * L.Kx;
        const int max_back = net->host_tables[conv_of_dev[l]].max_back;
        // pixel tile: a power of two between 16 and 1024, small enough to give about 256 work items
        int pt = WG;
        while (pt > 16 && (pt / 2 >= Pin || (long long)L.Mi * ((Pin + pt - 1) / pt) < 256)) pt /= 2;
        s.tw_log2 = ceil_log2(pt);
        s.n_tiles = (Pin + pt - 1) / pt;
        s.n_items = L.Mi * s.n_tiles;
        s.chunk = std::max(1, std::min({LDS_IN / ((L.Ho + 1) * (L.Wo + 1)), LDS_AUX / KK, std::max(1, max_back)}));
        (void)HW;
        // ... then adjust the weights of layer l one stage later
        pending_wgrad = l;
      } else {
        // first trainable layer: nothing to pull; adjust it together with whatever is pending
        if (pending_wgrad >= 0) { add_wgrad(pending_wgrad, 0); pending_wgrad = -1; }
        add_wgrad(l, 1);
      }
    }
  }
  if (pending_wgrad >= 0) { add_wgrad(pending_wgrad, 1); pending_wgrad = -1; }
  if (ns > 0) P.stages[ns - 1].barrier_after = 1;
  P.n_stages = ns;

  int rc = check_plan(net);
  if (rc) return rc;
  plan_flow(net);
  if (net->mode == CNN_MODE_RESIDENT && !net->flow_ok) net->mode = CNN_MODE_PERSISTENT;
  return CNN_OK;
}


// Resident mode: choose the team, lay out every rank's LDS (flow_plan, shared with the kernels that
// are compiled for fixed networks) and the exchange buffers.  Sets net->flow_ok; a network the mode
// cannot take keeps flow_ok = false with the reason in flow_why (not an error: the other modes
// still run it).
void plan_flow(cnn* net) {
  const ProgramDev& P = net->prog;
  FlowSpec& Z = net->flow;
  FlowPtrs& Q = net->flow_ptrs;
  std::memset(&Z, 0, sizeof(Z));
  std::memset(&Q, 0, sizeof(Q));
  net->flow_ok = false;
  net->flow_static_id = 0;
  net->special_active = false;
  auto no = [&](const std::string& why) { net->flow_why = why; };
  int n_conv = 0;
  while (n_conv < P.n_layers && P.layers[n_conv].kind == L_CONV) ++n_conv;
  const int n_fc = P.n_layers - n_conv;
  if (n_conv < 1) return no("resident mode needs at least one convolutional layer");
  if (n_conv > FLOW_MAX_CONV || n_fc > FLOW_MAX_FC || n_fc < 1)
    return no("resident mode takes at most " + std::to_string(FLOW_MAX_CONV) + " convolutional and " +
              std::to_string(FLOW_MAX_FC) + " fully connected layers");
  Z.n_conv = n_conv; Z.n_fc = n_fc; Z.n_classes = P.n_classes; Z.out_units = net->out_units;
  for (int l = 0; l < n_conv; ++l) {
    const LayerDev& L = P.layers[l];
    if (L.rect) return no("resident mode takes kernels, skipping factors and pooling rectangles with equal x and y values only");
    ConvSpec& C = Z.conv[l];
    C.Mi = L.Mi; C.Hi = L.Hi; C.Wi = L.Wi; C.Mo = L.Mo; C.Ho = L.Ho; C.Wo = L.Wo;
    C.K = L.K; C.S = L.S; C.Kp = L.Kp; C.Hp = L.Hp; C.Wp = L.Wp;
    C.max_conn = L.max_conn; C.max_back = net->host_tables[l].max_back; C.full_table = L.full_table;
  }
  for (int f = 0; f < n_fc; ++f) {
    const LayerDev& L = P.layers[n_conv + f];
    Z.fc[f].n_in = L.n_in; Z.fc[f].n_out = L.n_out; Z.fc[f].is_output = L.is_output;
  }
  switch (flow_plan(Z, net->team_ranks, net->team_stride, net->n_cu)) {
    case FLOW_OK: break;
    case FLOW_BAD_STRIDE: return no("team stride must be 1 or 8");
    case FLOW_TOO_LARGE: return no("a layer is too large for resident mode");
    case FLOW_NO_LDS: return no("the weights and maps one workgroup would hold exceed its LDS");
    default: return no("resident mode cannot run this network");
  }
  // pointers: layers, tables, exchange buffers
  tagged_t* xb = net->d_xbuf;
  size_t xoff = 0;
  auto xtake = [&](size_t words) { tagged_t* p = xb ? xb + xoff : nullptr; xoff += words; return p; };
  for (int l = 0; l < n_conv; ++l) {
    const LayerDev& L = P.layers[l];
    FlowConvPtrs& C = Q.conv[l];
    C.w = L.w; C.bias = L.bias; C.act = L.act; C.out = L.out; C.arg = L.arg; C.argyx = L.argyx; C.delta = L.delta;
    C.csr_ptr = L.csr_ptr; C.csr_idx = L.csr_idx; C.csc_ptr = L.csc_ptr; C.csc_j = L.csc_j; C.csc_slot = L.csc_slot;
    C.w_canon = L.w_canon; C.b_canon = L.b_canon;
    const size_t small = (size_t)L.Mo * L.Hp * L.Wp;
    C.x_out = (l + 1 < n_conv) ? xtake(2 * small) : nullptr;
    C.x_delta = (l >= 1) ? xtake(2 * small) : nullptr;
    C.x_yx = (l >= 1) ? xtake(2 * small) : nullptr;
    C.x_part = (l >= 1 && Z.conv[l].pull_shares > 1)
                   ? xtake((size_t)2 * L.Mi * (Z.conv[l].pull_shares - 1) * L.Hi * L.Wi) : nullptr;
    C.x_w = (l >= 1 && Z.stream) ? xtake((size_t)2 * net->host_tables[l].csr_idx.size() * (L.K * L.K + 4)) : nullptr;
  }
  for (int f = 0; f < n_fc; ++f) {
    const LayerDev& L = P.layers[n_conv + f];
    FlowFcPtrs& C = Q.fc[f];
    C.w = L.w; C.bias = L.bias; C.act = L.act; C.delta = L.delta; C.w_canon = L.w_canon; C.b_canon = L.b_canon;
    C.x_part = nullptr; C.x_dprev = nullptr;
    if (Z.fc[f].by_cols) {
      C.x_part = xtake((size_t)2 * std::min(Z.G, Z.fc[f].n_in) * Z.fc[f].n_out);
      C.x_dprev = xtake((size_t)2 * Z.fc[f].n_in);
    }
  }
  Q.xp = xtake((size_t)2 * Z.n_col_ranks * Z.fc[0].n_out);
  Q.xsum = xtake((size_t)2 * Z.fc[0].n_out);
  if (xoff > net->xbuf_words) return no("internal: exchange buffers exceed their workspace area");
  if (xb && !Q.xp) return no("internal: an exchange buffer was not laid out");
  net->flow_static_id = resident_static_id(Z);
  net->special_active = net->special_func != nullptr && std::memcmp(&Z, &net->special_plan, sizeof(FlowSpec)) == 0;
  net->flow_ok = true;
  net->flow_why.clear();
}

// Upload what plan() built.  Weights are zeroed.
int upload(cnn* net) {
  const ProgramDev& P = net->prog;
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  int conv_i = 0;
  for (int l = 0; l < P.n_layers; ++l) {
    const LayerDev& L = P.layers[l];
    if (L.kind != L_CONV) continue;
    const cnn::HostTable& T = net->host_tables[conv_i];
    const cnn::ConvBuf& b = net->conv_buf[conv_i];
    HIP_TRY(net, hipMemcpy(b.csr_ptr, T.csr_ptr.data(), T.csr_ptr.size() * 4, hipMemcpyHostToDevice));
    HIP_TRY(net, hipMemcpy(b.csr_idx, T.csr_idx.data(), T.csr_idx.size() * 4, hipMemcpyHostToDevice));
    HIP_TRY(net, hipMemcpy(b.csc_ptr, T.csc_ptr.data(), T.csc_ptr.size() * 4, hipMemcpyHostToDevice));
    HIP_TRY(net, hipMemcpy(b.csc_j, T.csc_j.data(), T.csc_j.size() * 4, hipMemcpyHostToDevice));
    HIP_TRY(net, hipMemcpy(b.csc_slot, T.csc_slot.data(), T.csc_slot.size() * 4, hipMemcpyHostToDevice));
    if (L.Kp == 1 && L.Kpx == 1) {  // no pooling: every neuron is its own winner
      std::vector<int> yx((size_t)L.Mo * L.Ho * L.Wo);
      for (int j = 0; j < L.Mo; ++j)
        for (int y = 0; y < L.Ho; ++y)
          for (int x = 0; x < L.Wo; ++x) yx[((size_t)j * L.Ho + y) * L.Wo + x] = (y << 16) | x;
      HIP_TRY(net, hipMemcpy(L.argyx, yx.data(), yx.size() * 4, hipMemcpyHostToDevice));
      HIP_TRY(net, hipMemset(L.arg, 0, yx.size()));
    }
    ++conv_i;
  }
  HIP_TRY(net, hipMemcpy(net->d_prog, &P, sizeof(P), hipMemcpyHostToDevice));
  HIP_TRY(net, hipMemcpy(net->d_flow_ptrs, &net->flow_ptrs, sizeof(FlowPtrs), hipMemcpyHostToDevice));
  HIP_TRY(net, hipMemset(net->d_xbuf, 0, net->xbuf_words * sizeof(tagged_t)));
  net->epoch = 0;
  HIP_TRY(net, hipMemset(net->d_weights, 0, net->n_weights_max * sizeof(float)));
  HIP_TRY(net, hipMemset(net->d_status, 0, sizeof(StatusDev)));
  return CNN_OK;
}

int rebuild(cnn* net) {
  int rc = plan(net);
  if (rc) return rc;
  return upload(net);
}

int check_status(cnn* net) {
  StatusDev s;
  HIP_TRY(net, hipMemcpy(&s, net->d_status, sizeof(s), hipMemcpyDeviceToHost));
  int rc = CNN_OK;
  if (s.abort_flag) rc = fail(&net->err, CNN_E_HIP, "a wait inside the persistent or resident kernel timed out; the weights are undefined");
  else if (s.bad_label) rc = fail(&net->err, CNN_E_ARG, "a label outside [0, classes) was met; that image was skipped");
  if (s.abort_flag || s.bad_label) {
    const float loss = s.loss;
    std::memset(&s, 0, sizeof(s));
    s.loss = loss;
    HIP_TRY(net, hipMemcpy(net->d_status, &s, sizeof(s), hipMemcpyHostToDevice));
  }
  return rc;
}

int sync_and_check(cnn* net) {
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  return check_status(net);
}

int persistent_grid(const cnn* net, int train) {
  if (net->grid_override > 0) return std::min(net->grid_override, net->n_cu * net->max_blocks_per_cu);
  int most = 1;
  for (int s = 0; s < net->prog.n_stages; ++s)
    if (train || !net->prog.stages[s].train_only) most = std::max(most, net->prog.stages[s].n_items);
  return std::max(1, std::min(most, net->n_cu));
}

void drop_stage_graphs(cnn* net) {
  if (net->graph_exec[0] || net->graph_exec[1]) (void)hipStreamSynchronize(net->stream);  // (replays may be in flight)
  for (int w = 0; w < 2; ++w) {
    if (net->graph_exec[w]) (void)hipGraphExecDestroy(net->graph_exec[w]);
    net->graph_exec[w] = nullptr;
    net->graph_built_for[w] = 0;
  }
}

// The stage launches of `images` consecutive images as a chain of kernel nodes behind one node that moves the
// call's image counter on; every stage node carries its image's place in the graph, the rest comes from *d_call.
int build_stage_graph(cnn* net, int which, int images, const RunArgs& a0) {
  const ProgramDev& P = net->prog;
  if (net->graph_exec[which]) { (void)hipGraphExecDestroy(net->graph_exec[which]); net->graph_exec[which] = nullptr; }
  hipGraph_t graph = nullptr;
  HIP_TRY(net, hipGraphCreate(&graph, 0));
  auto give_up = [&](hipError_t e, const char* what) { (void)hipGraphDestroy(graph); return hip_fail(net, e, what); };
  hipGraphNode_t prev = nullptr;
  auto add = [&](const void* fn, unsigned grid, unsigned block, void** params) -> hipError_t {
    hipKernelNodeParams kp;
    std::memset(&kp, 0, sizeof(kp));
    kp.func = const_cast<void*>(fn);
    kp.gridDim = dim3(grid); kp.blockDim = dim3(block); kp.sharedMemBytes = 0; kp.kernelParams = params; kp.extra = nullptr;
    hipGraphNode_t node = nullptr;
    hipError_t e = hipGraphAddKernelNode(&node, graph, prev ? &prev : nullptr, prev ? 1 : 0, &kp);
    prev = node;
    return e;
  };
  {
    CallArgs* d_call = net->d_call;
    int step = images;
    void* params[] = {(void*)&d_call, (void*)&step};
    hipError_t e = add(call_advance_kernel(), 1, 64, params);
    if (e != hipSuccess) return give_up(e, "graph node (image counter)");
  }
  const ProgramDev* d_prog = net->d_prog;
  StatusDev* d_status = net->d_status;
  for (int i = 0; i < images; ++i) {
    RunArgs b = a0;
    b.call = net->d_call; b.t_local = i;
    b.images = nullptr; b.labels = nullptr; b.probs_out = nullptr; b.grad_out = nullptr; b.n_images = 1;
    for (int s = 0; s < P.n_stages; ++s) {
      const Stage& st = P.stages[s];
      if (st.train_only && !which) continue;
      if (st.n_items <= 0) continue;
      int stage = s;
      void* params[] = {(void*)&d_prog, (void*)&stage, (void*)&d_status, (void*)&b};
      if (!st.barrier_after && s + 1 < P.n_stages && P.stages[s + 1].train_only == st.train_only && P.stages[s + 1].n_items > 0) {
        const Stage& nx = P.stages[s + 1];
        if (const void* fn = stage_pair_kernel(st.kind, nx.kind)) {
          hipError_t e = add(fn, (unsigned)(st.n_items + nx.n_items), WG, params);
          if (e != hipSuccess) return give_up(e, "graph node (pair of stages)");
          ++s;
          continue;
        }
      }
      const void* fn = stage_kernel(st.kind);
      if (!fn) return give_up(hipErrorInvalidValue, "graph node (unknown stage)");
      hipError_t e = add(fn, (unsigned)st.n_items, WG, params);
      if (e != hipSuccess) return give_up(e, "graph node (stage)");
    }
  }
  hipGraphExec_t exec = nullptr;
  hipError_t e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) return hip_fail(net, e, "hipGraphInstantiate");
  net->graph_exec[which] = exec;
  net->graph_built_for[which] = images;
  return CNN_OK;
}

// The resident kernel of this handle: the one loaded for its own network when the plan is still the one that was
// compiled for, else a compiled-in one (for a benchmark network, or the one that reads its plan).
static hipError_t launch_resident_of(cnn* net, int grid, size_t lds_bytes, const RunArgs& a) {
  if (!net->special_active)
    return launch_resident(net->flow_static_id, grid, lds_bytes, net->stream, net->flow, net->d_flow_ptrs, net->d_status, a);
  RunArgs args = a;
  FlowSpec plan = net->flow;
  const FlowPtrs* d_ptrs = net->d_flow_ptrs;
  StatusDev* d_status = net->d_status;
  void* params[] = {(void*)&plan, (void*)&d_ptrs, (void*)&d_status, (void*)&args};
  return hipModuleLaunchCooperativeKernel(net->special_func, (unsigned)grid, 1, 1, WG, 1, 1, (unsigned)lds_bytes, net->stream, params);
}

int run(cnn* net, const RunArgs& a0) {
  RunArgs a = a0;
  a.spin_limit = net->spin_limit;
  a.barrier_kind = net->barrier_kind;
  const ProgramDev& P = net->prog;
  if (net->mode == CNN_MODE_RESIDENT) {
    const unsigned long long n = (unsigned long long)a.n_images;
    if (n >= (1ull << 31)) return fail(&net->err, CNN_E_ARG, "too many images in one call");
    if (((net->epoch + n) >> 32) != (net->epoch >> 32)) {
      // the 32-bit tags would wrap inside this call: start a fresh range on cleared buffers
      net->epoch = ((net->epoch >> 32) + 1) << 32;
      HIP_TRY(net, hipStreamSynchronize(net->stream));
      HIP_TRY(net, hipMemset(net->d_xbuf, 0, net->xbuf_words * sizeof(tagged_t)));
    }
    const int grid = net->flow.G * net->flow.stride;
    const size_t lds_bytes = (size_t)net->flow.lds_floats * sizeof(float);
    HIP_TRY(net, launch_reset_status(net->stream, net->d_status, 0));
    if (!P.has_frontend) {
      a.epoch_base = (unsigned int)net->epoch;
      net->epoch += n;
      HIP_TRY(net, launch_resident_of(net, grid, lds_bytes, a));
      return CNN_OK;
    }
    // fixed front-end: computed for FE_BATCH images at a time by all compute units, outside the
    // on-line chain; the resident kernel then trains on its outputs
    const size_t fe_sz = (size_t)P.fe.n_filters * P.fe.H * P.fe.W;
    const int items = (int)((fe_sz + WG - 1) / WG);
    for (unsigned long long t0 = 0; t0 < n; t0 += FE_BATCH) {
      const int nb = (int)std::min<unsigned long long>(FE_BATCH, n - t0);
      HIP_TRY(net, launch_frontend_batch(net->stream, net->d_prog, a0.images + t0 * a0.image_stride, a0.image_stride,
                                         nb, items, net->d_fe_batch));
      RunArgs b = a;
      b.images = net->d_fe_batch;
      b.image_stride = (long long)fe_sz;
      b.labels = a.labels ? a.labels + t0 : nullptr;
      b.probs_out = a.probs_out ? a.probs_out + t0 * P.n_classes : nullptr;
      b.n_images = nb;
      b.epoch_base = (unsigned int)net->epoch;
      net->epoch += (unsigned long long)nb;
      HIP_TRY(net, launch_resident_of(net, grid, lds_bytes, b));
      if (t0 + nb >= n)  // parity tap: layer 0 of the last image
        HIP_TRY(net, hipMemcpyAsync(net->d_fe_out, net->d_fe_batch + (size_t)(nb - 1) * fe_sz, fe_sz * sizeof(float),
                                    hipMemcpyDeviceToDevice, net->stream));
    }
    return CNN_OK;
  }
  if (net->mode == CNN_MODE_PERSISTENT) {
    HIP_TRY(net, launch_reset_status(net->stream, net->d_status, 0));
    bool mm = false;
    for (int s = 0; s < P.n_stages; ++s) mm = mm || P.stages[s].kind >= ST_CONV_FWD_MFMA;
    HIP_TRY(net, launch_persistent(persistent_grid(net, a.train), mm, net->stream, net->d_prog, net->d_status, a));
    return CNN_OK;
  }
  const long long n = a.n_images;
  long long t_first = 0;
  const int GB = net->graph_images;
  if (GB > 0 && a.labels && !a.grad_out && n >= 2 * GB) {
    // whole graphs of GB images first; what is left over is launched stage by stage below
    const int which = a.train ? 1 : 0;
    if (!net->graph_exec[which] || net->graph_built_for[which] != GB) {
      int rc = build_stage_graph(net, which, GB, a);
      if (rc) return rc;
    }
    CallArgs c;
    c.images = a.images; c.labels = a.labels; c.probs_out = a.probs_out; c.image_stride = a.image_stride;
    c.t0 = -(long long)GB; c.lr = a.lr; c.train = a.train;
    HIP_TRY(net, launch_call_set(net->stream, net->d_call, c));
    const long long n_graphs = n / GB;
    for (long long g = 0; g < n_graphs; ++g) HIP_TRY(net, hipGraphLaunch(net->graph_exec[which], net->stream));
    t_first = n_graphs * GB;
  }
  for (long long t = t_first; t < n; ++t) {
    RunArgs b = a;
    b.images = a.images + t * a.image_stride;
    b.labels = a.labels ? a.labels + t : nullptr;
    b.probs_out = a.probs_out ? a.probs_out + t * P.n_classes : nullptr;
    b.n_images = 1;
    for (int s = 0; s < P.n_stages; ++s) {
      const Stage& st = P.stages[s];
      if (st.train_only && !a.train) continue;
      if (!st.barrier_after && s + 1 < P.n_stages && P.stages[s + 1].train_only == st.train_only) {
        // the next stage does not depend on this one: both in one launch, where a kernel for the pair exists
        const Stage& nx = P.stages[s + 1];
        bool done = false;
        HIP_TRY(net, launch_stage_pair(st.kind, st.n_items, nx.kind, nx.n_items, net->stream, net->d_prog, s,
                                       net->d_status, b, &done));
        if (done) { ++s; continue; }
      }
      HIP_TRY(net, launch_stage(st.kind, st.n_items, net->stream, net->d_prog, s, net->d_status, b));
    }
  }
  return CNN_OK;
}

}  // namespace

// ---- batched forward pass ------------------------------------------------------------------
namespace {

struct BatchStep {
  BatchGemm g;
  BatchPool pool;     // used when g.fuse == 0
  BatchPack pack;
  size_t wt_off = 0;  // floats from the start of the scratch
  size_t wt_floats = 0;
  size_t out_per_image = 0;
};
struct BatchPlan {
  std::vector<BatchStep> steps;
  size_t wt_total = 0, sums_per_image = 0, act_per_image = 0, fe_per_image = 0;
  size_t floats(size_t batch) const {
    return wt_total + batch * (sums_per_image + 2 * act_per_image + fe_per_image) + 4 * 64;
  }
};

size_t up64(size_t x) { return (x + 63) / 64 * 64; }

// Shape of every layer's matrix product, tile choice and LDS budget.  Returns 0 or an error code.
int batch_plan(cnn* net, size_t batch, BatchPlan& B) {
  const ProgramDev& P = net->prog;
  constexpr size_t LDS_FLOATS = 20000;      // 78 KB per workgroup: two workgroups per compute unit
  constexpr size_t LDS_FLOATS_BIG = 38000;  // large input maps: one workgroup per compute unit
  B = BatchPlan();
  for (int l = 0; l < P.n_layers; ++l) {
    const LayerDev& L = P.layers[l];
    BatchStep st;
    BatchGemm& g = st.g;
    std::memset(&g, 0, sizeof(g));
    int Kp = 1, Kpx = 1, Ho = 1, Hp = 1, Wp = 1;
    if (L.kind == L_CONV) {
      g.Mi = L.Mi; g.Hi = L.Hi; g.Wi = L.Wi; g.K = L.K; g.Kx = L.Kx; g.stride = L.S + 1; g.stride_x = L.Sx + 1;
      g.Mo = L.Mo; g.Wo = L.Wo;
      g.P = L.Ho * L.Wo; Ho = L.Ho; Kp = L.Kp; Kpx = L.Kpx; Hp = L.Hp; Wp = L.Wp;
    } else {  // a fully connected layer: n_in maps of one pixel, K = 1
      g.Mi = L.n_in; g.Hi = 1; g.Wi = 1; g.K = 1; g.Kx = 1; g.stride = 1; g.stride_x = 1; g.Mo = L.n_out; g.Wo = 1; g.P = 1;
    }
    const bool pooled = Kp * Kpx > 1;
    // map tiles per workgroup: the choice that pads the fewest maps, the larger on a tie; tiles of 16 maps only
    // where they pad fewer than tiles of 32 do (40 maps: 48 rows instead of 64), at least two of them a workgroup
    // (an operand fetched from the staged images should feed several instructions)
    int best_pad = 0;
    g.TR = 32;
    for (int mt : {4, 2, 1}) {
      const int pad = (g.Mo + 32 * mt - 1) / (32 * mt) * (32 * mt);
      if (!best_pad || pad < best_pad) { best_pad = pad; g.MT = mt; }
    }
    for (int mt : {6, 5, 4, 3, 2}) {
      const int pad = (g.Mo + 16 * mt - 1) / (16 * mt) * (16 * mt);
      if (pad < best_pad) { best_pad = pad; g.MT = mt; g.TR = 16; }
    }
    g.MoPad = best_pad;
    const int KK = g.K * g.Kx, HiWi = g.Hi * g.Wi;
    // input maps per chunk: as many as the LDS budget takes; when that leaves several chunks,
    // prefer a chunk that also fits the prefetch registers (16 + 48 floats per thread), unless
    // such a chunk would be too short to hide anything behind.  One-pixel maps (fully connected
    // layers) take a power of two, so that staging finds image and offset by shifting.
    int ic = 0, ic_pre = 0;
    auto fit = [&](int cols_per_image, size_t budget) {
      g.n_img_max = (int)std::min<size_t>(std::max<size_t>(batch, 1), (size_t)((128 - 1 + cols_per_image - 1) / cols_per_image + 1));
      ic = 0; ic_pre = 0;
      for (int c = 1; c <= g.Mi; ++c) {
        const size_t in_f = (size_t)g.n_img_max * c * HiWi, w_f = (size_t)(c * KK + 1) * g.MT * g.TR;
        if (in_f + 3 + w_f + (size_t)c * KK + (g.TR == 32 ? 9 : 20) > budget) break;
        if (HiWi == 1 && c < g.Mi && (c & (c - 1)) != 0) continue;
        ic = c;
        if (in_f <= 16 * 256 && w_f <= 48 * 256) ic_pre = c;
      }
    };
    // Pooling inside the product: when the whole k range is one chunk, a column is a pooled pixel
    // and the wavefront walks the Kp x Kpx members of its window one after the other, keeping the
    // running maximum in registers; the full-resolution sums then never reach memory.
    g.Kp = 1; g.Kpx = 1;
    bool pool_inside = false;
    if (pooled) {
      fit(Hp * Wp, LDS_FLOATS);
      if (ic == g.Mi) { g.Kp = Kp; g.Kpx = Kpx; g.P = Hp * Wp; g.Wo = Wp; pool_inside = true; }
    }
    if (!pool_inside) {
      fit(g.P, LDS_FLOATS);
      if (ic == 0) fit(g.P, LDS_FLOATS_BIG);
    }
    if (ic == 0)
      return fail(&net->err, CNN_E_SHAPE, "batched forward pass: one input map of a layer (times the images a "
                                          "workgroup touches) exceeds the LDS budget");
    g.prefetch = 0;
    if (ic < g.Mi && ic_pre * KK >= 96) { ic = ic_pre; g.prefetch = 1; }
    g.IC = ic;
    // few columns and a long k range (fully connected layers, deep layers on small maps): the k
    // range is cut into slices, one workgroup each, until some 512 workgroups are in flight
    const int n_chunks = (g.Mi + ic - 1) / ic;
    const size_t wgs = ((batch * g.P + 127) / 128) * (size_t)(g.MoPad / (g.TR * g.MT));
    int ks = 1;
    if (wgs < 512 && n_chunks > 1) ks = (int)std::min<size_t>((size_t)n_chunks, (512 + wgs - 1) / wgs);
    g.chunks_per_slice = (n_chunks + ks - 1) / ks;
    g.KS = (n_chunks + g.chunks_per_slice - 1) / g.chunks_per_slice;
    g.slice_stride = (long long)(batch * g.Mo * g.P);
    g.fuse = ((pooled && !pool_inside) || g.KS > 1) ? 0 : (L.is_output ? 2 : 1);
    g.bias = L.bias;
    g.in_stride = (long long)g.Mi * HiWi;
    g.out_stride = (long long)g.Mo * g.P;
    st.wt_floats = up64((size_t)g.Mi * KK * g.MoPad);
    st.wt_off = B.wt_total;
    B.wt_total += st.wt_floats;
    BatchPack& k = st.pack;
    std::memset(&k, 0, sizeof(k));
    k.w = L.w; k.csr_ptr = L.csr_ptr; k.csr_idx = L.csr_idx;
    k.is_fc = L.kind != L_CONV; k.full_table = L.full_table; k.Mi = g.Mi; k.Mo = g.Mo; k.K = g.K; k.Kx = g.Kx; k.n_in = L.n_in;
    k.MoPad = g.MoPad;
    if (L.kind == L_CONV) {
      int ci = 0;
      for (int q = 0; q < l; ++q) ci += P.layers[q].kind == L_CONV;
      k.total = (long long)net->host_tables[ci].csr_idx.size() * KK;
    } else {
      k.total = (long long)L.n_in * L.n_out;
    }
    BatchPool& q = st.pool;
    std::memset(&q, 0, sizeof(q));
    q.bias = L.bias; q.Mo = g.Mo; q.Ho = Ho; q.Wo = (L.kind == L_CONV) ? L.Wo : 1; q.Kp = Kp; q.Kpx = Kpx; q.Hp = Hp; q.Wp = Wp;
    q.n_slices = g.KS; q.slice_stride = g.slice_stride; q.act = L.is_output ? 0 : 1;
    st.out_per_image = pooled ? (size_t)g.Mo * Hp * Wp : (size_t)g.Mo * g.P;
    if (g.fuse == 0) B.sums_per_image = std::max(B.sums_per_image, up64((size_t)g.KS * g.Mo * g.P));
    // (g.P is Ho * Wo whenever fuse == 0 with pooling: pooling inside the product always has fuse != 0)
    B.act_per_image = std::max(B.act_per_image, up64(st.out_per_image));
    B.steps.push_back(st);
  }
  if (P.has_frontend) B.fe_per_image = up64((size_t)P.fe.n_filters * P.fe.H * P.fe.W);
  return CNN_OK;
}

}  // namespace


extern "C" {

int cnn_arch_info(const char* arch, int32_t* n_layers, int32_t* info, int32_t max_layers) {
  std::vector<ArchLayer> A;
  int rc = parse_arch(arch, A, nullptr);
  if (rc) return rc;
  if (n_layers) *n_layers = (int32_t)A.size();
  if (info)
    for (size_t l = 0; l < A.size() && (int32_t)l < max_layers; ++l) {
      int32_t* o = info + 6 * l;
      o[0] = A[l].kind; o[1] = A[l].maps; o[2] = A[l].h; o[3] = A[l].w; o[4] = A[l].K; o[5] = A[l].S;
    }
  return CNN_OK;
}

int cnn_arch_info_xy(const char* arch, int32_t* n_layers, int32_t* info, int32_t max_layers) {
  std::vector<ArchLayer> A;
  int rc = parse_arch(arch, A, nullptr);
  if (rc) return rc;
  if (n_layers) *n_layers = (int32_t)A.size();
  if (info)
    for (size_t l = 0; l < A.size() && (int32_t)l < max_layers; ++l) {
      int32_t* o = info + 8 * l;
      o[0] = A[l].kind; o[1] = A[l].maps; o[2] = A[l].h; o[3] = A[l].w; o[4] = A[l].K; o[5] = A[l].S;
      o[6] = A[l].Kx; o[7] = A[l].Sx;
    }
  return CNN_OK;
}

int cnn_workspace_bytes(const char* arch, size_t* bytes) {
  if (!bytes) return fail(nullptr, CNN_E_ARG, "bytes is NULL");
  cnn tmp;
  int rc = parse_arch(arch, tmp.arch, nullptr);
  if (rc) return rc;
  *bytes = carve(&tmp, nullptr);
  for (size_t l = 1; l < tmp.arch.size(); ++l)
    if (tmp.arch[l].kind == CNN_LAYER_CONV)
      tmp.tables.emplace_back((size_t)tmp.arch[l].maps * tmp.arch[l - 1].maps, (uint8_t)1);
  rc = plan(&tmp);  // shapes the kernels cannot take are refused here, without a device
  if (rc) g_err = tmp.err;
  return rc;
}

static int plan_to_text(const ProgramDev& P, char* buf, size_t n) {
  static const char* names[] = {"?", "frontend", "conv_fwd", "fc_fwd", "head", "fc_bwd", "conv_bwd", "conv_wgrad", "conv_mfma", "conv_epi",
                                "conv_bwd_mfma", "conv_bwd_epi", "conv_wgrad_mfma"};
  std::string out;
  char line[256];
  for (int s = 0; s < P.n_stages; ++s) {
    const Stage& st = P.stages[s];
    std::snprintf(line, sizeof line, "%2d %-10s layer=%d items=%d barrier=%d train_only=%d rows=%d tiles=%d chunk=%d tw=%d ppt=%d rpw=%d cm=%d\n",
                  s, names[st.kind], st.layer, st.n_items, st.barrier_after, st.train_only, st.tile_rows, st.n_tiles,
                  st.chunk, 1 << st.tw_log2, st.pix_per_thread, st.rows_per_wg, 1 << st.cm_log2);
    out += line;
  }
  std::snprintf(buf, n, "%s", out.c_str());
  return CNN_OK;
}

int cnn_plan_text(const char* arch, char* buf, size_t n) {
  if (!buf || n == 0) return fail(nullptr, CNN_E_ARG, "buf is NULL");
  cnn tmp;
  int rc = parse_arch(arch, tmp.arch, nullptr);
  if (rc) return rc;
  carve(&tmp, nullptr);
  for (size_t l = 1; l < tmp.arch.size(); ++l)
    if (tmp.arch[l].kind == CNN_LAYER_CONV)
      tmp.tables.emplace_back((size_t)tmp.arch[l].maps * tmp.arch[l - 1].maps, (uint8_t)1);
  rc = plan(&tmp);
  if (rc) { g_err = tmp.err; return rc; }
  return plan_to_text(tmp.prog, buf, n);
}

int cnn_get_plan_text(const cnn_t* net, char* buf, size_t n) {
  if (!net || !buf || n == 0) return CNN_E_ARG;
  return plan_to_text(net->prog, buf, n);
}

int cnn_create(const char* arch, void* d_workspace, size_t bytes, void* hip_stream, cnn_t** out) {
  if (!out) return fail(nullptr, CNN_E_ARG, "out is NULL");
  *out = nullptr;
  cnn* net = new cnn;
  int rc = parse_arch(arch, net->arch, &net->err);
  if (rc) { delete net; return rc; }
  const size_t need = carve(net, nullptr);
  if (!d_workspace || bytes < need || ((uintptr_t)d_workspace & 255)) {
    delete net;
    return fail(nullptr, CNN_E_WORKSPACE, "workspace must be 256-byte aligned device memory of at least " +
                                              std::to_string(need) + " bytes");
  }
  carve(net, d_workspace);
  net->stream = (hipStream_t)hip_stream;
  for (size_t l = 1; l < net->arch.size(); ++l)
    if (net->arch[l].kind == CNN_LAYER_CONV)
      net->tables.emplace_back((size_t)net->arch[l].maps * net->arch[l - 1].maps, (uint8_t)1);
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&net->n_cu, hipDeviceAttributeMultiprocessorCount, dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&net->coop_ok, hipDeviceAttributeCooperativeLaunch, dev);
  if (e != hipSuccess) { rc = hip_fail(nullptr, e, "device query"); delete net; return rc; }
  net->device = dev;
  net->max_blocks_per_cu = std::max(1, persistent_max_blocks_per_cu());
  rc = rebuild(net);
  if (rc) { g_err = net->err; delete net; return rc; }
  *out = net;
  return CNN_OK;
}

void cnn_destroy(cnn_t* net) {
  if (!net) return;
  (void)hipStreamSynchronize(net->stream);
  if (net->special_module) (void)hipModuleUnload(net->special_module);
  drop_stage_graphs(net);
  delete net;
}

int cnn_set_connection_table(cnn_t* net, int conv_index, const uint8_t* host_table) {
  if (!net || !host_table) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (conv_index < 0 || conv_index >= (int)net->tables.size()) return fail(&net->err, CNN_E_ARG, "no such convolutional layer");
  int seen = 0, mo = 0, mi = 0;
  for (size_t l = 1; l < net->arch.size(); ++l)
    if (net->arch[l].kind == CNN_LAYER_CONV && seen++ == conv_index) { mo = net->arch[l].maps; mi = net->arch[l - 1].maps; }
  std::vector<uint8_t> t((size_t)mo * mi);
  for (int j = 0; j < mo; ++j) {
    bool any = false;
    for (int i = 0; i < mi; ++i) { t[(size_t)j * mi + i] = host_table[(size_t)j * mi + i] ? 1 : 0; any |= t[(size_t)j * mi + i] != 0; }
    if (!any) return fail(&net->err, CNN_E_ARG, "output map " + std::to_string(j) + " has no input map");
  }
  net->tables[conv_index] = t;
  return rebuild(net);
}

int cnn_set_fixed_frontend(cnn_t* net, int n_filters, int K, int n_src_channels, const float* host_filters,
                           const int32_t* host_src_channel) {
  if (!net || !host_filters || !host_src_channel) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (n_filters != net->arch[0].maps) return fail(&net->err, CNN_E_ARG, "n_filters must equal the input maps of the architecture");
  if (K < 1 || K > MAX_FRONTEND_K || n_src_channels < 1) return fail(&net->err, CNN_E_ARG, "bad front-end size");
  for (int f = 0; f < n_filters; ++f)
    if (host_src_channel[f] < 0 || host_src_channel[f] >= n_src_channels) return fail(&net->err, CNN_E_ARG, "source channel out of range");
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  net->fe_n = n_filters; net->fe_K = K; net->fe_src_n = n_src_channels;
  net->fe_filters.assign(host_filters, host_filters + (size_t)n_filters * K * K);
  net->fe_src.assign(host_src_channel, host_src_channel + n_filters);
  HIP_TRY(net, hipMemcpy(net->d_fe_filters, net->fe_filters.data(), net->fe_filters.size() * 4, hipMemcpyHostToDevice));
  HIP_TRY(net, hipMemcpy(net->d_fe_src, net->fe_src.data(), net->fe_src.size() * 4, hipMemcpyHostToDevice));
  return rebuild(net);
}

size_t cnn_num_weights(const cnn_t* net) { return net ? net->n_weights : 0; }
size_t cnn_image_size(const cnn_t* net) { return net ? net->image_size : 0; }
int cnn_num_layers(const cnn_t* net) { return net ? (int)net->arch.size() : 0; }
int cnn_num_classes(const cnn_t* net) { return net ? net->n_classes : 0; }

int cnn_layer_info(const cnn_t* net, int layer, int32_t* o) {
  if (!net || !o || layer < 0 || layer >= (int)net->arch.size()) return CNN_E_ARG;
  const ArchLayer& a = net->arch[layer];
  o[0] = a.kind; o[1] = a.maps; o[2] = a.h; o[3] = a.w; o[4] = a.K; o[5] = a.S;
  return CNN_OK;
}

int cnn_layer_info_xy(const cnn_t* net, int layer, int32_t* o) {
  if (!net || !o || layer < 0 || layer >= (int)net->arch.size()) return CNN_E_ARG;
  const ArchLayer& a = net->arch[layer];
  o[0] = a.kind; o[1] = a.maps; o[2] = a.h; o[3] = a.w; o[4] = a.K; o[5] = a.S; o[6] = a.Kx; o[7] = a.Sx;
  return CNN_OK;
}

int cnn_get_weights(cnn_t* net, float* host_dst, size_t n) {
  if (!net || !host_dst) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (n != net->n_weights) return fail(&net->err, CNN_E_ARG, "weight count mismatch");
  int rc = sync_and_check(net);
  HIP_TRY(net, hipMemcpy(host_dst, net->d_weights, n * sizeof(float), hipMemcpyDeviceToHost));
  return rc;
}

int cnn_set_weights(cnn_t* net, const float* host_src, size_t n) {
  if (!net || !host_src) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (n != net->n_weights) return fail(&net->err, CNN_E_ARG, "weight count mismatch");
  int rc = sync_and_check(net);
  HIP_TRY(net, hipMemcpy(net->d_weights, host_src, n * sizeof(float), hipMemcpyHostToDevice));
  return rc;
}

int cnn_forward(cnn_t* net, const float* d_image, float* d_probs) {
  return cnn_forward_many(net, d_image, 1, d_probs);
}

int cnn_forward_many(cnn_t* net, const float* d_images, size_t n, float* d_probs) {
  if (!net || !d_images) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (n == 0) return CNN_OK;
  RunArgs a;
  std::memset(&a, 0, sizeof(a));
  a.images = d_images; a.probs_out = d_probs; a.n_images = (long long)n; a.image_stride = (long long)net->image_size;
  a.label_imm = -1; a.train = 0;
  return run(net, a);
}

int cnn_train_step(cnn_t* net, const float* d_image, int32_t label, float lr) {
  if (!net || !d_image) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (label < 0 || label >= net->n_classes) return fail(&net->err, CNN_E_ARG, "label out of range");
  RunArgs a;
  std::memset(&a, 0, sizeof(a));
  a.images = d_image; a.n_images = 1; a.image_stride = (long long)net->image_size;
  a.label_imm = label; a.train = 1; a.lr = lr;
  return run(net, a);
}

int cnn_train_many(cnn_t* net, const float* d_images, const int32_t* d_labels, size_t n, float lr) {
  if (!net || !d_images || !d_labels) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (n == 0) return CNN_OK;
  RunArgs a;
  std::memset(&a, 0, sizeof(a));
  a.images = d_images; a.labels = d_labels; a.n_images = (long long)n; a.image_stride = (long long)net->image_size;
  a.train = 1; a.lr = lr;
  return run(net, a);
}

int cnn_set_mode(cnn_t* net, int mode) {
  if (!net) return CNN_E_ARG;
  if (mode != CNN_MODE_STAGES && mode != CNN_MODE_PERSISTENT && mode != CNN_MODE_RESIDENT)
    return fail(&net->err, CNN_E_ARG, "unknown mode");
  if (mode != CNN_MODE_STAGES && !net->coop_ok) return fail(&net->err, CNN_E_STATE, "device does not support cooperative launches");
  if (mode == CNN_MODE_RESIDENT && !net->flow_ok) return fail(&net->err, CNN_E_STATE, net->flow_why);
  const bool replan = (mode == CNN_MODE_STAGES) != (net->mode == CNN_MODE_STAGES);
  if (replan) HIP_TRY(net, hipStreamSynchronize(net->stream));
  const int old_mode = net->mode;
  net->mode = mode;
  if (replan) {
    // the stage-launch mode pulls the deltas of wide layers on the matrix cores, the other modes do
    // not: the stage list differs; weights, tables and everything else on the device stay
    int rc = plan(net);
    if (rc) { net->mode = old_mode; return rc; }
    net->mode = mode;
    HIP_TRY(net, hipMemcpy(net->d_prog, &net->prog, sizeof(ProgramDev), hipMemcpyHostToDevice));
      HIP_TRY(net, hipMemcpy(net->d_flow_ptrs, &net->flow_ptrs, sizeof(FlowPtrs), hipMemcpyHostToDevice));
  }
  return CNN_OK;
}

int cnn_mode_supported(cnn_t* net, int mode) {
  if (!net) return 0;
  if (mode == CNN_MODE_STAGES) return 1;
  if (mode == CNN_MODE_PERSISTENT) return net->coop_ok ? 1 : 0;
  if (mode == CNN_MODE_RESIDENT) return (net->coop_ok && net->flow_ok) ? 1 : 0;
  return 0;
}

int cnn_get_mode(const cnn_t* net) { return net ? net->mode : CNN_E_ARG; }

// ---- a resident kernel compiled for the handle's own network -----------------------------------------
// The text of a header that gives cnn355_flowspec.h the network of this handle as StaticSpec<FLOW_SPECIAL_ID>:
// the same inputs plan_flow() hands the planner, so the compiler arrives at the same plan.
int cnn_resident_spec_source(const cnn_t* net, char* buf, size_t n) {
  if (!net) return fail(nullptr, CNN_E_ARG, "net is NULL");
  if (!net->flow_ok) return fail(nullptr, CNN_E_STATE, "resident mode cannot run this network: " + net->flow_why);
  const FlowSpec& Z = net->flow;
  std::string t = "// written by cnn_resident_spec_source\n";
  t += "constexpr FlowSpec flow_special_spec() {\n  FlowSpec Z{};\n";
  auto set = [&](const std::string& name, int v) { t += "  Z." + name + " = " + std::to_string(v) + ";\n"; };
  set("n_conv", Z.n_conv); set("n_fc", Z.n_fc); set("n_classes", Z.n_classes); set("out_units", Z.out_units);
  for (int l = 0; l < Z.n_conv; ++l) {
    const ConvSpec& C = Z.conv[l];
    const std::string c = "conv[" + std::to_string(l) + "].";
    set(c + "Mi", C.Mi); set(c + "Hi", C.Hi); set(c + "Wi", C.Wi); set(c + "Mo", C.Mo); set(c + "Ho", C.Ho); set(c + "Wo", C.Wo);
    set(c + "K", C.K); set(c + "S", C.S); set(c + "Kp", C.Kp); set(c + "Hp", C.Hp); set(c + "Wp", C.Wp);
    set(c + "max_conn", C.max_conn); set(c + "max_back", C.max_back); set(c + "full_table", C.full_table);
  }
  for (int f = 0; f < Z.n_fc; ++f) {
    const std::string c = "fc[" + std::to_string(f) + "].";
    set(c + "n_in", Z.fc[f].n_in); set(c + "n_out", Z.fc[f].n_out); set(c + "is_output", Z.fc[f].is_output);
  }
  t += "  flow_plan(Z, " + std::to_string(net->team_ranks) + ", " + std::to_string(net->team_stride) + ", " +
       std::to_string(net->n_cu > 0 ? net->n_cu : 256) + ");\n  return Z;\n}\n";
  t += "template <>\nstruct StaticSpec<FLOW_SPECIAL_ID> {\n  static constexpr FlowSpec value = flow_special_spec();\n};\n";
  if (buf && n > 0) {
    const size_t k = std::min(n - 1, t.size());
    std::memcpy(buf, t.data(), k);
    buf[k] = 0;
  }
  return (int)t.size();
}

int cnn_load_resident_code(cnn_t* net, const char* path) {
  if (!net || !path) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (!net->d_status) return fail(&net->err, CNN_E_STATE, "cnn_load_resident_code: the handle has no workspace");
  if (!net->flow_ok) return fail(&net->err, CNN_E_STATE, "resident mode cannot run this network: " + net->flow_why);
  int device = -1;
  HIP_TRY(net, hipGetDevice(&device));
  if (device != net->device)
    return fail(&net->err, CNN_E_STATE, "cnn_load_resident_code: the current device is not the one the network was created on");
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  hipModule_t mod = nullptr;
  if (hipModuleLoad(&mod, path) != hipSuccess) {
    (void)hipGetLastError();
    return fail(&net->err, CNN_E_ARG, std::string("cannot load a gfx950 code object from ") + path);
  }
  auto drop = [&](int code, const std::string& why) { (void)hipModuleUnload(mod); return fail(&net->err, code, why); };
  hipDeviceptr_t d_plan = nullptr;
  size_t bytes = 0;
  if (hipModuleGetGlobal(&d_plan, &bytes, mod, "cnn355_special_plan") != hipSuccess || bytes != sizeof(FlowSpec)) {
    (void)hipGetLastError();
    return drop(CNN_E_ARG, "the code object holds no plan of this library's layout (built from other sources?)");
  }
  FlowSpec plan;
  if (hipMemcpy(&plan, d_plan, sizeof(FlowSpec), hipMemcpyDeviceToHost) != hipSuccess) {
    (void)hipGetLastError();
    return drop(CNN_E_HIP, "cannot read the plan out of the code object");
  }
  if (std::memcmp(&plan, &net->flow, sizeof(FlowSpec)) != 0)
    return drop(CNN_E_STATE, "the code object was compiled for another network, table, output variant or team than this "
                             "handle has now");
  hipFunction_t f = nullptr;
  if (hipModuleGetFunction(&f, mod, "_ZN6cnn35510k_residentILi99EEEvNS_8FlowSpecEPKNS_8FlowPtrsEPNS_9StatusDevENS_7RunArgsE") != hipSuccess) {
    (void)hipGetLastError();
    return drop(CNN_E_ARG, "the code object holds no resident kernel");
  }
  if (net->special_module) (void)hipModuleUnload(net->special_module);
  net->special_module = mod;
  net->special_func = f;
  net->special_plan = plan;
  net->special_active = true;
  return CNN_OK;
}

int cnn_resident_code_active(const cnn_t* net) { return (net && net->flow_ok && net->special_active) ? 1 : 0; }

// development aid, not part of the public header: which compiled-in network the resident plan equals (0: none)
int cnn355_resident_static_id(const cnn_t* net) { return net ? net->flow_static_id : -1; }
// development aid: 1 when the resident plan streams the inputs of the layers above the first (0: they stay in LDS)
int cnn355_resident_streams(const cnn_t* net) { return (net && net->flow_ok) ? net->flow.stream : 0; }
// development aid: workgroups in the resident plan's team (0 when the network cannot run in resident mode)
int cnn355_resident_ranks(const cnn_t* net) { return (net && net->flow_ok) ? net->flow.G : 0; }
// development aid, host only (no device is touched): the resident plan of an architecture as text.  fan_in > 0
// gives every convolutional layer above the first a table in which output map j reads the input maps
// j, j + 1, ..., j + fan_in - 1 (mod M_i); fan_in = -d stands for M_i / d of them in every layer.  One line per number ("name value"), per layer ("conv l name value ...")
// and per LDS region of a rank ("region name first_float floats"); a region's size is restated here from its
// documented shape, not taken from the planner.
static int plan_only(cnn& tmp, const char* arch, int fan_in, int n_ranks, int xcd_stride) {
  int rc = parse_arch(arch, tmp.arch, nullptr);
  if (rc) return rc;
  carve(&tmp, nullptr);
  for (size_t l = 1; l < tmp.arch.size(); ++l)
    if (tmp.arch[l].kind == CNN_LAYER_CONV) {
      const int Mo = tmp.arch[l].maps, Mi = tmp.arch[l - 1].maps;
      const int fan = fan_in < 0 ? std::max(1, Mi / -fan_in) : fan_in;
      const bool sparse = fan > 0 && fan < Mi && !tmp.tables.empty();
      tmp.tables.emplace_back((size_t)Mo * Mi, (uint8_t)(sparse ? 0 : 1));
      if (sparse)
        for (int j = 0; j < Mo; ++j)
          for (int k = 0; k < fan; ++k) tmp.tables.back()[(size_t)j * Mi + (j + k) % Mi] = 1;
    }
  tmp.team_ranks = n_ranks;
  tmp.team_stride = xcd_stride;
  rc = plan(&tmp);
  if (rc) g_err = tmp.err;
  return rc;
}

// development aid, host only: cnn_resident_spec_source for an architecture without a handle (tables as in
// cnn355_resident_plan_text), so that code objects can be compiled where there is no GPU
int cnn355_resident_spec_source_for(const char* arch, int fan_in, int n_ranks, int xcd_stride, char* buf, size_t n) {
  cnn tmp;
  const int rc = plan_only(tmp, arch, fan_in, n_ranks, xcd_stride);
  if (rc) return rc;
  return cnn_resident_spec_source(&tmp, buf, n);
}

int cnn355_resident_plan_text(const char* arch, int fan_in, int n_ranks, int xcd_stride, char* buf, size_t n) {
  if (!buf || n == 0) return fail(nullptr, CNN_E_ARG, "buf is NULL");
  cnn tmp;
  int rc = plan_only(tmp, arch, fan_in, n_ranks, xcd_stride);
  if (rc) return rc;
  std::string t;
  auto num = [&](const char* name, long long v) { t += std::string(name) + " " + std::to_string(v) + "\n"; };
  if (!tmp.flow_ok) {
    t = "unsupported " + tmp.flow_why + "\n";
  } else {
    const FlowSpec& Z = tmp.flow;
    num("G", Z.G); num("stride", Z.stride); num("n_conv", Z.n_conv); num("n_fc", Z.n_fc);
    num("n_col_ranks", Z.n_col_ranks); num("fc1_owned", Z.fc1_owned); num("lds_floats", Z.lds_floats); num("lds_floats_max", FLOW_LDS_FLOATS_MAX);
    num("scratch_floats", Z.scratch_floats); num("defer", Z.defer); num("static_id", tmp.flow_static_id);
    num("stream", Z.stream);
    num("workgroup", WG); num("share_min_macs", FLOW_SHARE_MIN_MACS);
    auto region = [&](const std::string& name, long long off, long long floats) {
      t += "region " + name + " " + std::to_string(off) + " " + std::to_string(floats) + "\n";
    };
    long long act = 1, dall = 1;
    for (int l = 0; l < Z.n_conv; ++l) {
      const ConvSpec& C = Z.conv[l];
      const long long KK = C.K * C.K, HW = C.Hp * C.Wp;
      const std::string c = "conv" + std::to_string(l) + ".";
      t += "conv " + std::to_string(l);
      const std::pair<const char*, int> f[] = {
          {"Mi", C.Mi}, {"Hi", C.Hi}, {"Wi", C.Wi}, {"Mo", C.Mo}, {"Ho", C.Ho}, {"Wo", C.Wo}, {"K", C.K}, {"S", C.S},
          {"Kp", C.Kp}, {"Hp", C.Hp}, {"Wp", C.Wp}, {"max_conn", C.max_conn}, {"max_back", C.max_back},
          {"full_table", C.full_table}, {"n_own", C.n_own}, {"n_own_below", C.n_own_below},
          {"pull_shares", C.pull_shares}, {"back_pitch", C.back_pitch}, {"wgrad_R_log2", C.wgrad_R_log2},
          {"pull_chunk", C.pull_chunk}, {"fwd_strip", C.fwd_strip}, {"fwd_rows", C.fwd_rows},
          {"pull_strip", C.pull_strip}, {"pull_rows", C.pull_rows}, {"in_chunk", C.in_chunk}, {"pull_slots", C.pull_slots}};
      for (const auto& kv : f) t += std::string(" ") + kv.first + " " + std::to_string(kv.second);
      t += "\n";
      if (!(Z.stream && l >= 1)) region(c + "in", C.o_in, (long long)C.Mi * C.Hi * C.Wi);
      region(c + "wf", C.o_wf, (long long)C.n_own * C.max_conn * KK);
      region(c + "bf", C.o_bf, C.n_own);
      region(c + "cidx", C.o_cidx, (long long)C.n_own * C.max_conn);
      region(c + "ncf", C.o_ncf, C.n_own);
      if (l >= 1) {
        region(c + "wb", C.o_wb, (long long)C.n_own_below * C.back_pitch * KK);
        region(c + "bj", C.o_bj, (long long)C.n_own_below * C.back_pitch);
        region(c + "ncb", C.o_ncb, C.n_own_below);
        dall = std::max(dall, (long long)C.Mo * HW);
      }
      region(c + "pool", C.o_pool, C.n_own * HW);
      region(c + "yx", C.o_yx, C.n_own * HW);
      region(c + "delta", C.o_delta, C.n_own * HW);
      region(c + "dact", C.o_dact, C.n_own * HW);
      if (C.o_tab_fwd >= 0) region(c + "tab_fwd", C.o_tab_fwd, 3 * WG);
      if (C.o_tab_pull >= 0) region(c + "tab_pull", C.o_tab_pull, 3 * WG);
      act = std::max(act, (long long)C.n_own * C.Ho * C.Wo);
    }
    const ConvSpec& Cl = Z.conv[Z.n_conv - 1];
    for (int f = 0; f < Z.n_fc; ++f) {
      const FcSpec& Q = Z.fc[f];
      const std::string c = "fc" + std::to_string(f) + ".";
      t += "fc " + std::to_string(f) + " n_in " + std::to_string(Q.n_in) + " n_out " + std::to_string(Q.n_out) +
           " by_cols " + std::to_string(Q.by_cols) + " n_own " + std::to_string(Q.n_own) + "\n";
      region(c + "w", Q.o_w, f == 0 ? (long long)Cl.n_own * Cl.Hp * Cl.Wp * Q.n_out
                             : Q.by_cols ? (long long)Q.n_own * Q.n_out : (long long)Q.n_out * Q.n_in);
      region(c + "b", Q.o_b, Q.n_out);
      region(c + "act", Q.o_act, Q.n_out);
      region(c + "delta", Q.o_delta, Q.n_out);
      region(c + "dact", Q.o_dact, Q.n_out);
    }
    region("act", Z.o_act, act);
    // (the partial sums reach up to the next region: what they need is for the reader to work out)
    if (!Z.stream) region("part", Z.o_part, Z.o_dall - Z.o_part);
    if (Z.n_conv > 1) {
      region("dall", Z.o_dall, dall);
      region("yxall", Z.o_yxall, dall);
    }
    if (Z.defer && Z.n_conv > 1) region("prev", Z.o_prev, (long long)Z.conv[1].n_own_below * Z.conv[1].Hi * Z.conv[1].Wi);
    region("scratch", Z.o_scratch, Z.scratch_floats);
  }
  if (t.size() + 1 > n) return fail(nullptr, CNN_E_ARG, "buffer too small for the plan text");
  std::memcpy(buf, t.c_str(), t.size() + 1);
  return CNN_OK;
}

// development aid: how many ranks share the delta pull into one input map of the resident plan's conv layer l
int cnn355_resident_pull_shares(const cnn_t* net, int l) {
  if (!net || !net->flow_ok || l < 0 || l >= net->flow.n_conv) return -1;
  return net->flow.conv[l].pull_shares;
}

int cnn_set_team(cnn_t* net, int n_ranks, int xcd_stride) {
  if (!net || n_ranks < 0 || (xcd_stride != 0 && xcd_stride != 1 && xcd_stride != 8)) return CNN_E_ARG;
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  net->team_ranks = n_ranks;
  net->team_stride = xcd_stride;
  plan_flow(net);
  if (net->d_flow_ptrs)
    HIP_TRY(net, hipMemcpy(net->d_flow_ptrs, &net->flow_ptrs, sizeof(FlowPtrs), hipMemcpyHostToDevice));
  if (net->mode == CNN_MODE_RESIDENT && !net->flow_ok) {
    net->mode = CNN_MODE_PERSISTENT;
    return fail(&net->err, CNN_E_STATE, net->flow_why);
  }
  return CNN_OK;
}

int cnn_set_matrix_cores(cnn_t* net, int on) {
  if (!net) return CNN_E_ARG;
  if ((on != 0) == (net->use_mfma != 0)) return CNN_OK;
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  net->use_mfma = on ? 1 : 0;
  // re-plan the stages only: tables, weights and everything else on the device stay as they are
  int rc = plan(net);
  if (rc) return rc;
  HIP_TRY(net, hipMemcpy(net->d_prog, &net->prog, sizeof(ProgramDev), hipMemcpyHostToDevice));
  HIP_TRY(net, hipMemcpy(net->d_flow_ptrs, &net->flow_ptrs, sizeof(FlowPtrs), hipMemcpyHostToDevice));
  return CNN_OK;
}

int cnn_set_output_units(cnn_t* net, int kind) {
  if (!net || (kind != CNN_OUTPUT_SOFTMAX_XENT && kind != CNN_OUTPUT_TANH_SQERR)) return CNN_E_ARG;
  if (kind == net->out_units) return CNN_OK;
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  net->out_units = kind;
  // re-plan: the descriptors carry the kind; weights, tables and buffers stay as they are
  int rc = plan(net);
  if (rc) return rc;
  HIP_TRY(net, hipMemcpy(net->d_prog, &net->prog, sizeof(ProgramDev), hipMemcpyHostToDevice));
  HIP_TRY(net, hipMemcpy(net->d_flow_ptrs, &net->flow_ptrs, sizeof(FlowPtrs), hipMemcpyHostToDevice));
  return CNN_OK;
}

int cnn_get_output_units(const cnn_t* net) { return net ? net->out_units : CNN_E_ARG; }

int cnn_set_launch_graph(cnn_t* net, int images_per_graph) {
  if (!net || images_per_graph < 0 || images_per_graph > 1024) return fail(net ? &net->err : nullptr, CNN_E_ARG, "images_per_graph must lie in [0, 1024]");
  if (images_per_graph != net->graph_images) drop_stage_graphs(net);
  net->graph_images = images_per_graph;
  return CNN_OK;
}

int cnn_set_grid(cnn_t* net, int n_workgroups) {
  if (!net || n_workgroups < 0) return CNN_E_ARG;
  net->grid_override = n_workgroups;
  return CNN_OK;
}

int cnn_set_barrier(cnn_t* net, int kind) {
  if (!net || (kind != 0 && kind != 1)) return CNN_E_ARG;
  net->barrier_kind = kind;
  return CNN_OK;
}

int cnn_set_spin_limit(cnn_t* net, unsigned int polls) {
  if (!net) return CNN_E_ARG;
  net->spin_limit = polls;
  return CNN_OK;
}

int cnn_synchronize(cnn_t* net) {
  if (!net) return CNN_E_ARG;
  return sync_and_check(net);
}

int cnn_get_activation(cnn_t* net, int layer, float* host_dst) {
  if (!net || !host_dst) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (layer < 0 || layer >= (int)net->arch.size()) return fail(&net->err, CNN_E_ARG, "no such layer");
  int rc = sync_and_check(net);
  const ArchLayer& a = net->arch[layer];
  const size_t n = (size_t)a.maps * a.h * a.w;
  const float* src = nullptr;
  if (layer == 0) {
    if (!net->fe_n) return fail(&net->err, CNN_E_STATE, "layer 0 is the caller's image unless a front-end is set");
    src = net->d_fe_out;
  } else {
    const LayerDev& L = net->prog.layers[net->dev_of_arch[layer]];
    src = (a.kind == CNN_LAYER_POOL) ? L.out : L.act;
  }
  HIP_TRY(net, hipMemcpy(host_dst, src, n * sizeof(float), hipMemcpyDeviceToHost));
  return rc;
}

int cnn_get_delta(cnn_t* net, int layer, float* host_dst) {
  if (!net || !host_dst) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (layer < 1 || layer >= (int)net->arch.size() || net->arch[layer].kind == CNN_LAYER_POOL)
    return fail(&net->err, CNN_E_ARG, "deltas exist for convolutional and fully connected layers");
  int rc = sync_and_check(net);
  const ArchLayer& a = net->arch[layer];
  const LayerDev& L = net->prog.layers[net->dev_of_arch[layer]];
  if (a.kind == CNN_LAYER_FC) {
    HIP_TRY(net, hipMemcpy(host_dst, L.delta, (size_t)a.maps * sizeof(float), hipMemcpyDeviceToHost));
    return rc;
  }
  // scatter the winners' deltas back to the full-resolution map (index work only)
  const size_t small = (size_t)L.Mo * L.Hp * L.Wp, full = (size_t)L.Mo * L.Ho * L.Wo;
  std::vector<float> d(small);
  std::vector<int> yx(small);
  HIP_TRY(net, hipMemcpy(d.data(), L.delta, small * sizeof(float), hipMemcpyDeviceToHost));
  HIP_TRY(net, hipMemcpy(yx.data(), L.argyx, small * sizeof(int), hipMemcpyDeviceToHost));
  std::fill(host_dst, host_dst + full, 0.f);
  for (int j = 0; j < L.Mo; ++j)
    for (int q = 0; q < L.Hp * L.Wp; ++q) {
      const int v = yx[(size_t)j * L.Hp * L.Wp + q];
      const int y = v >> 16, x = v & 0xffff;
      if (y < 0 || y >= L.Ho || x >= L.Wo) continue;  // no forward pass has filled the winners yet
      host_dst[((size_t)j * L.Ho + y) * L.Wo + x] = d[(size_t)j * L.Hp * L.Wp + q];
    }
  return rc;
}

int cnn_get_argmax(cnn_t* net, int pool_layer, uint8_t* host_dst) {
  if (!net || !host_dst) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (pool_layer < 1 || pool_layer >= (int)net->arch.size() || net->arch[pool_layer].kind != CNN_LAYER_POOL)
    return fail(&net->err, CNN_E_ARG, "not a max-pooling layer");
  int rc = sync_and_check(net);
  const ArchLayer& a = net->arch[pool_layer];
  const LayerDev& L = net->prog.layers[net->dev_of_arch[pool_layer]];
  HIP_TRY(net, hipMemcpy(host_dst, L.arg, (size_t)a.maps * a.h * a.w, hipMemcpyDeviceToHost));
  return rc;
}

int cnn_get_loss(cnn_t* net, float* host_loss) {
  if (!net || !host_loss) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  StatusDev s;
  HIP_TRY(net, hipMemcpy(&s, net->d_status, sizeof(s), hipMemcpyDeviceToHost));
  *host_loss = s.loss;
  return check_status(net);
}

int cnn_get_stage_times(cnn_t* net, float* host_us, int max_stages, int* n_stages) {
  if (!net || !host_us || !n_stages) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  StatusDev s;
  HIP_TRY(net, hipMemcpy(&s, net->d_status, sizeof(s), hipMemcpyDeviceToHost));
  const int n = net->prog.n_stages;
  *n_stages = n;
  unsigned long long prev = s.stamps[0];
  for (int k = 0; k < n && k < max_stages; ++k) {
    const unsigned long long a = s.stamps[1 + 2 * k], b = s.stamps[2 + 2 * k];
    host_us[2 * k] = (a >= prev) ? (float)(a - prev) * 0.01f : 0.f;
    host_us[2 * k + 1] = (b >= a) ? (float)(b - a) * 0.01f : 0.f;
    if (b >= prev) prev = b;
  }
  return CNN_OK;
}

int cnn_debug_gradients(cnn_t* net, const float* d_image, int32_t label, float* host_grad) {
  if (!net || !d_image || !host_grad) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (label < 0 || label >= net->n_classes) return fail(&net->err, CNN_E_ARG, "label out of range");
  RunArgs a;
  std::memset(&a, 0, sizeof(a));
  a.images = d_image; a.n_images = 1; a.image_stride = (long long)net->image_size;
  a.label_imm = label; a.train = 1; a.lr = 0.f; a.grad_out = net->d_grad;
  int rc = run(net, a);
  if (rc) return rc;
  rc = sync_and_check(net);
  HIP_TRY(net, hipMemcpy(host_grad, net->d_grad, net->n_weights * sizeof(float), hipMemcpyDeviceToHost));
  return rc;
}

// development aid, not part of the public header: the raw device timestamps (100 MHz ticks) of the last call
int cnn355_read_status_stamps(cnn_t* net, unsigned long long* out, int n) {
  if (!net || !out) return CNN_E_ARG;
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  StatusDev s;
  HIP_TRY(net, hipMemcpy(&s, net->d_status, sizeof(s), hipMemcpyDeviceToHost));
  for (int i = 0; i < n && i < 2 * MAX_STAGES + 2; ++i) out[i] = s.stamps[i];
  return CNN_OK;
}

int cnn_measure_crossing(cnn_t* net, int n_ranks, int words_per_rank, int rounds, float* host_us) {
  if (!net || !host_us) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument");
  if (!net->coop_ok) return fail(&net->err, CNN_E_STATE, "device does not support cooperative launches");
  if (n_ranks < 2 || n_ranks > net->n_cu || words_per_rank < 1 || rounds < 1 || rounds > (1 << 20))
    return fail(&net->err, CNN_E_ARG, "cnn_measure_crossing: 2 to one rank per compute unit, at least one word and one round");
  if (2ull * n_ranks * words_per_rank > net->xbuf_words)
    return fail(&net->err, CNN_E_WORKSPACE, "cnn_measure_crossing: the network's exchange buffers hold " +
                std::to_string(net->xbuf_words / 2 / n_ranks) + " words per rank for this many ranks");
  const unsigned long long n = (unsigned long long)rounds + 1;
  HIP_TRY(net, hipStreamSynchronize(net->stream));
  if (((net->epoch + n) >> 32) != (net->epoch >> 32)) {
    net->epoch = ((net->epoch >> 32) + 1) << 32;
    HIP_TRY(net, hipMemset(net->d_xbuf, 0, net->xbuf_words * sizeof(tagged_t)));
  }
  HIP_TRY(net, launch_reset_status(net->stream, net->d_status, 0));
  const int stride = (n_ranks <= net->n_cu / 8) ? 8 : 1;
  HIP_TRY(net, launch_crossing_probe(n_ranks, stride, net->stream, net->d_xbuf, words_per_rank, rounds,
                                     (unsigned int)net->epoch, net->spin_limit, net->d_status));
  net->epoch += n;
  int rc = sync_and_check(net);
  if (rc) return rc;
  StatusDev s;
  HIP_TRY(net, hipMemcpy(&s, net->d_status, sizeof(s), hipMemcpyDeviceToHost));
  *host_us = (float)((double)(s.stamps[1] - s.stamps[0]) * 0.01 / rounds);
  return CNN_OK;
}

int cnn_measure_launch(cnn_t* net, int rounds, float* host_us) {
  if (!net || !host_us || rounds < 1) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument or no rounds");
  hipEvent_t e0, e1;
  HIP_TRY(net, hipEventCreate(&e0));
  HIP_TRY(net, hipEventCreate(&e1));
  for (int k = 0; k < 20; ++k) HIP_TRY(net, launch_empty(net->stream, net->d_status));
  HIP_TRY(net, hipEventRecord(e0, net->stream));
  for (int k = 0; k < rounds; ++k) HIP_TRY(net, launch_empty(net->stream, net->d_status));
  HIP_TRY(net, hipEventRecord(e1, net->stream));
  HIP_TRY(net, hipEventSynchronize(e1));
  float ms = 0.f;
  HIP_TRY(net, hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *host_us = ms * 1e3f / (float)rounds;
  return CNN_OK;
}

// development aid, not part of the public header: in-item timestamps (zeros unless built with CNN355_STAMPS)
void cnn355_read_stamps(unsigned long long* out64) { cnn355::read_dbg(out64); }

const char* cnn_last_error(const cnn_t* net) { return net ? net->err.c_str() : g_err.c_str(); }

int cnn_forward_batch_scratch_bytes(cnn_t* net, size_t batch, size_t* bytes) {
  if (!net || !bytes || batch == 0) return fail(net ? &net->err : nullptr, CNN_E_ARG, "NULL argument or batch of 0");
  BatchPlan B;
  int rc = batch_plan(net, batch, B);
  if (rc) return rc;
  *bytes = B.floats(batch) * sizeof(float);
  return CNN_OK;
}

int cnn_deform_images(void* hip_stream, const float* d_src, size_t n_src, float* d_dst, size_t n, int C, int H, int W,
                      const cnn_deform_params* p, uint64_t seed, uint64_t first_index,
                      const int32_t* d_src_index, float* d_displacement) {
  if (n == 0) return CNN_OK;
  if (n_src == 0 || n_src > 0x7fffffffull || (!d_src_index && n > n_src))
    return fail(nullptr, CNN_E_ARG, "cnn_deform_images: more outputs than source images and no index list, or no source images");
  if (!d_src || !d_dst || !p) return fail(nullptr, CNN_E_ARG, "cnn_deform_images: NULL argument");
  if (d_src == d_dst) return fail(nullptr, CNN_E_ARG, "cnn_deform_images: source and destination must not overlap");
  if (C < 1 || H < 1 || W < 1 || (long long)H * (W | 1) > DEFORM_MAX_PIXELS || C > 1024)
    return fail(nullptr, CNN_E_SHAPE, "cnn_deform_images: rows x (columns rounded up to odd) at most 9312 (96 x 96), 1 to 1024 maps per image");
  if (n > (size_t)1 << 40) return fail(nullptr, CNN_E_ARG, "cnn_deform_images: too many images");
  const float ranges[6] = {p->max_translation, p->max_rotation, p->max_scaling, p->max_shear, p->sigma, p->fill};
  for (float r : ranges)
    if (!std::isfinite(r)) return fail(nullptr, CNN_E_ARG, "cnn_deform_images: a parameter is not finite");
  if (!std::isfinite(p->alpha)) return fail(nullptr, CNN_E_ARG, "cnn_deform_images: a parameter is not finite");
  if (p->max_translation < 0 || p->max_rotation < 0 || p->max_scaling < 0 || p->max_shear < 0 || p->sigma < 0)
    return fail(nullptr, CNN_E_ARG, "cnn_deform_images: a range or sigma is negative");
  if (p->max_scaling >= 1.0f) return fail(nullptr, CNN_E_ARG, "cnn_deform_images: max_scaling must be below 1");
  if (p->sigma > 16.0f) return fail(nullptr, CNN_E_ARG, "cnn_deform_images: sigma above 16 pixels");
  DeformJob J;
  J.src = d_src; J.dst = d_dst; J.disp = d_displacement; J.src_index = d_src_index;
  J.n = (long long)n; J.n_src = (long long)n_src; J.C = C; J.H = H; J.W = W;
  J.max_tx = (double)p->max_translation * W;
  J.max_ty = (double)p->max_translation * H;
  J.max_rot = (double)p->max_rotation * 3.14159265358979323846 / 180.0;
  J.max_shear = p->max_shear; J.max_scale = p->max_scaling; J.alpha = p->alpha; J.fill = p->fill;
  J.seed = seed; J.first_index = first_index;
  J.R = -1;
  for (float& t : J.taps) t = 0.f;
  if (p->sigma > 0.f && p->alpha != 0.f) {
    const double sg = p->sigma;
    const int R = (int)std::ceil(3.0 * sg);
    double g[2 * DEFORM_MAX_R + 1], sum = 0;
    for (int i = -R; i <= R; ++i) sum += g[i + R] = std::exp(-(double)i * i / (2.0 * sg * sg));
    for (int i = 0; i <= 2 * R; ++i) J.taps[i] = (float)(g[i] / sum);
    J.R = R;
  }
  hipError_t e = launch_deform((hipStream_t)hip_stream, J);
  if (e != hipSuccess) return fail(nullptr, CNN_E_HIP, std::string("cnn_deform_images: ") + hipGetErrorString(e));
  return CNN_OK;
}

// tap_step >= 0 (parity tap): the pass stops behind that trainable layer and its outputs for the n <= batch
// images, [image][out_per_image], are copied to host_tap; d_probs is not written then.
static int forward_batch_impl(cnn_t* net, const float* d_images, size_t n, float* d_probs, void* d_scratch,
                              size_t scratch_bytes, size_t batch, int tap_step, float* host_tap, size_t* tap_per_image) {
  if (!net) return fail(nullptr, CNN_E_ARG, "NULL handle");
  if (n == 0) return CNN_OK;
  if (!d_images || (!d_probs && tap_step < 0) || !d_scratch || batch == 0) return fail(&net->err, CNN_E_ARG, "NULL argument or batch of 0");
  if (((uintptr_t)d_scratch & 255u) != 0) return fail(&net->err, CNN_E_ARG, "scratch must be 256-byte aligned");
  BatchPlan B;
  int rc = batch_plan(net, batch, B);
  if (rc) return rc;
  for (const BatchStep& st : B.steps) {
    const unsigned long long lim = (1ull << 31) - 256;
    const unsigned long long b = batch;
    if (b * (unsigned long long)st.g.P >= lim || b * (unsigned long long)st.g.out_stride >= lim ||
        b * (unsigned long long)st.g.in_stride >= lim || (unsigned long long)st.wt_floats >= lim)
      return fail(&net->err, CNN_E_ARG, "batch too large: the layer inputs and outputs of one batch must stay below 2^31 floats each");
  }
  if (net->prog.has_frontend && (unsigned long long)batch * net->image_size >= (1ull << 31) - 256)
    return fail(&net->err, CNN_E_ARG, "batch too large: the images of one batch must stay below 2^31 floats");
  if (scratch_bytes < B.floats(batch) * sizeof(float))
    return fail(&net->err, CNN_E_WORKSPACE, "scratch smaller than cnn_forward_batch_scratch_bytes says");
  if (tap_step >= 0 && (tap_step >= (int)B.steps.size() || n > batch || !host_tap))
    return fail(&net->err, CNN_E_ARG, "no such trainable layer, more images than one batch, or no buffer");
  const ProgramDev& P = net->prog;
  float* base = (float*)d_scratch;
  float* d_sums = base + B.wt_total;
  float* d_act[2] = {d_sums + batch * B.sums_per_image, d_sums + batch * (B.sums_per_image + B.act_per_image)};
  float* d_fe = d_act[1] + batch * B.act_per_image;
  // the weights as the products read them: one [k][map] matrix per layer, from their present values
  for (BatchStep& st : B.steps) {
    st.pack.wt = base + st.wt_off;
    HIP_TRY(net, launch_batch_pack(net->stream, st.pack, (long long)st.wt_floats));
  }
  const size_t fe_sz = P.has_frontend ? (size_t)P.fe.n_filters * P.fe.H * P.fe.W : 0;
  for (size_t t0 = 0; t0 < n; t0 += batch) {
    const size_t nb = std::min(batch, n - t0);
    const float* in = d_images + t0 * net->image_size;
    long long in_stride = (long long)net->image_size;
    if (P.has_frontend) {
      HIP_TRY(net, launch_frontend_batch(net->stream, net->d_prog, in, in_stride, (int)nb, (int)((fe_sz + WG - 1) / WG), d_fe));
      in = d_fe;
      in_stride = (long long)fe_sz;
    }
    int cur = 0;
    for (size_t s = 0; s < B.steps.size(); ++s) {
      BatchStep& st = B.steps[s];
      BatchGemm g = st.g;
      g.in = in; g.in_stride = in_stride; g.wt = base + st.wt_off; g.N = (long long)nb * g.P;
      float* out = d_act[cur];
      if (g.fuse == 0) {
        g.out = d_sums;
        HIP_TRY(net, launch_batch_gemm(net->stream, g));
        BatchPool q = st.pool;
        q.sums = d_sums; q.out = out; q.total = (long long)nb * q.Mo * q.Hp * q.Wp;
        HIP_TRY(net, launch_batch_pool(net->stream, q));
      } else {
        g.out = out;
        HIP_TRY(net, launch_batch_gemm(net->stream, g));
      }
      in = out;
      in_stride = (long long)st.out_per_image;
      cur ^= 1;
      if ((int)s == tap_step) {
        HIP_TRY(net, hipStreamSynchronize(net->stream));
        HIP_TRY(net, hipMemcpy(host_tap, out, nb * st.out_per_image * sizeof(float), hipMemcpyDeviceToHost));
        if (tap_per_image) *tap_per_image = st.out_per_image;
        return CNN_OK;
      }
    }
    HIP_TRY(net, launch_batch_outputs(net->stream, in, d_probs + t0 * P.n_classes, (long long)nb, P.n_classes, net->out_units));
  }
  return CNN_OK;
}

int cnn_forward_batch(cnn_t* net, const float* d_images, size_t n, float* d_probs, void* d_scratch,
                      size_t scratch_bytes, size_t batch) {
  return forward_batch_impl(net, d_images, n, d_probs, d_scratch, scratch_bytes, batch, -1, nullptr, nullptr);
}

int cnn_debug_forward_batch_layer(cnn_t* net, const float* d_images, size_t n, int trainable_layer, float* host_out,
                                  size_t* host_floats_per_image, void* d_scratch, size_t scratch_bytes) {
  return forward_batch_impl(net, d_images, n, nullptr, d_scratch, scratch_bytes, n, trainable_layer, host_out,
                            host_floats_per_image);
}

}  // extern "C"

// ---- the batched forward pass for callers that cannot allocate ------------------------------------
// cnn_forward_batch takes its scratch memory from the caller.  This variant takes it from an array that
// is part of the library's device image instead, so that the call allocates nothing anywhere.  In host
// code the array's name only stands for the symbol: the address of the memory on the device that is
// current comes from hipGetSymbolAddress, once per device (every device holds its own copy), and only
// that address is ever used.
namespace {
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)CNN_FORWARD_BATCH_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
void* g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// the array's address on the current device (asked for once per device), or NULL with *err set
void* static_scratch_ptr(hipError_t* err, int* device) {
  *err = hipGetDevice(device);
  if (*err != hipSuccess) return nullptr;
  if (*device < 0 || *device >= STATIC_SCRATCH_MAX_DEVICES) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[*device]) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || !p) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
    g_scratch_ptr[*device] = p;
  }
  return g_scratch_ptr[*device];
}
}  // namespace

extern "C" int cnn_forward_batch_static(cnn_t* net, const float* d_images, size_t n, float* d_probs, size_t batch) {
  if (!net) return fail(nullptr, CNN_E_ARG, "NULL handle");
  if (n == 0) return CNN_OK;
  if (!d_images || !d_probs || batch == 0) return fail(&net->err, CNN_E_ARG, "NULL argument or batch of 0");
  size_t need = 0;
  int rc = cnn_forward_batch_scratch_bytes(net, batch, &need);
  if (rc) return rc;
  if (need > STATIC_SCRATCH_BYTES)
    return fail(&net->err, CNN_E_WORKSPACE, "cnn_forward_batch_static: a batch of " + std::to_string(batch) + " images needs " +
                std::to_string(need) + " bytes of scratch, the library's own array holds " +
                std::to_string(STATIC_SCRATCH_BYTES) + ": use a smaller batch, or cnn_forward_batch with memory of the caller's");
  hipError_t e = hipSuccess;
  int device = -1;
  void* ptr = static_scratch_ptr(&e, &device);
  if (!ptr) return hip_fail(net, e, "cnn_forward_batch_static: address of the scratch array");
  if (device != net->device)
    return fail(&net->err, CNN_E_STATE, "cnn_forward_batch_static: the current device is not the one the network was created on");
  return cnn_forward_batch(net, d_images, n, d_probs, ptr, STATIC_SCRATCH_BYTES, batch);
}
