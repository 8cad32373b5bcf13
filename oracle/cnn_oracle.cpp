// CPU oracle for online back-propagation training of the CNN variant of
// Ciresan et al., "High-Performance Neural Networks for Visual Object
// Classification" (IDSIA TR 01-11, 2011).
//
// THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
// transcription of the definitions (nested loops, no tiling, no fusion).  Only
// the tests, the smoke check and the CPU-baseline leg of the benchmark may
// call it; the GPU library shares no code with it and never falls back to it.
//
// Every routine names the passage of the paper it follows.  Where the paper is
// silent the reading taken is stated in the comment.
//
// Scalar type: `double` is the truth used for parity and finite differences;
// `float` exists only so the same loops can be timed as a CPU baseline.
//
// Parity pins (tests that do not need a GPU): output-size formula against the
// worked examples the paper prints (Sec. 2.2 Eq. 1, Fig. 2 caption, Sec. 4.3
// layer list), convolution against a library conv2d and against special cases,
// max-pool against brute force, pull form against push form (Sec. 3.3), every
// gradient against central finite differences (the paper's own check, Sec. 4),
// whole network against an autograd library in double.

#include <algorithm>
#include <cctype>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum Kind { K_INPUT = 0, K_CONV = 1, K_POOL = 2, K_FC = 3 };

enum Err {
  E_OK = 0,
  E_SYNTAX = -1,
  E_SHAPE = -2,
  E_ARG = -3,
};

// Scaled hyperbolic tangent of Sec. 4: y(a) = 1.7159 tanh(0.6666 a), constants
// exactly as printed.
constexpr double ACT_A = 1.7159;
constexpr double ACT_B = 0.6666;

template <class T> inline T scaled_tanh(T a) { return T(ACT_A) * std::tanh(T(ACT_B) * a); }
// dy/da written in terms of the output y:  A*B*(1 - tanh^2) = A*B - (B/A) y^2.
template <class T> inline T act_deriv_from_output(T y) {
  return T(ACT_A * ACT_B) - T(ACT_B / ACT_A) * y * y;
}

// ---------------------------------------------------------------------------
// Shapes
// ---------------------------------------------------------------------------

// Output map size of a convolutional layer, Sec. 2.2 Eq. (1):
//   M^n = (M^{n-1} - K^n) / (S^n + 1) + 1.
// The paper writes a plain fraction; where it is not integral we take the
// floor, which follows from Sec. 2.2's rule that a kernel position counts only
// when the whole kernel lies inside the input map.  Returns <= 0 when the
// kernel does not fit.
int conv_out_size(int m_prev, int k, int s) {
  if (m_prev < k) return 0;
  return (m_prev - k) / (s + 1) + 1;
}

struct Layer {
  int kind = K_INPUT;
  int maps = 0, h = 0, w = 0;  // output of this layer (FC: maps = neurons, h = w = 1)
  int ky = 0, kx = 0;          // conv kernel / pool rectangle
  int sy = 0, sx = 0;          // skipping factors (stride = s + 1), conv only
  // conv only: conn[j] = ascending list of input maps feeding output map j
  // (one row of the connection matrix C^n of Sec. 3.1).
  std::vector<std::vector<int>> conn;
  size_t b_off = 0, w_off = 0;  // offsets into the canonical weight vector
  size_t n_weights = 0;         // bias + kernels of this layer
};

// ---------------------------------------------------------------------------
// Layer operations (free functions, each the definition written out)
// ---------------------------------------------------------------------------

// Convolutional layer forward, Sec. 2.2 and Sec. 3.2: every output neuron
// starts from the bias of its map, adds, over all connected input maps and all
// kernel taps, weight times the input under the tap (the kernel lies fully
// inside the input; consecutive outputs are S+1 input pixels apart), then goes
// through the scaled tanh.  No kernel flip: the receptive field of output x is
// inputs x(S+1) .. x(S+1)+K-1 (inequalities of Sec. 3.3).
// w holds, for j ascending and i in conn[j] ascending, a ky*kx row-major block.
template <class T>
void conv_forward(const T* in, int mi, int hi, int wi, const T* bias, const T* w,
                  const std::vector<std::vector<int>>& conn, int ky, int kx, int sy, int sx,
                  int ho, int wo, bool apply_act, T* out) {
  (void)mi;
  const int mo = (int)conn.size();
  std::vector<size_t> first(mo, 0);
  size_t run = 0;
  for (int j = 0; j < mo; ++j) { first[j] = run; run += conn[j].size(); }
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (int j = 0; j < mo; ++j) {
    for (int y = 0; y < ho; ++y)
      for (int x = 0; x < wo; ++x) {
        T sum = bias ? bias[j] : T(0);
        for (size_t c = 0; c < conn[j].size(); ++c) {
          const int i = conn[j][c];
          const T* wk = w + (first[j] + c) * (size_t)(ky * kx);
          const T* im = in + (size_t)i * hi * wi;
          for (int a = 0; a < ky; ++a)
            for (int b = 0; b < kx; ++b)
              sum += wk[a * kx + b] * im[(size_t)(y * (sy + 1) + a) * wi + (x * (sx + 1) + b)];
        }
        out[((size_t)j * ho + y) * wo + x] = apply_act ? scaled_tanh(sum) : sum;
      }
  }
}

// Max-pooling forward, Sec. 2.3: maximum over non-overlapping ky x kx
// rectangles.  The index of the winner is kept for the backward pass:
// arg = dy*kx + dx of the first maximum met in a row-major scan (strict >);
// the paper does not say how ties are broken.
template <class T>
void maxpool_forward(const T* in, int m, int hi, int wi, int ky, int kx, T* out, uint8_t* arg) {
  const int ho = hi / ky, wo = wi / kx;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (int j = 0; j < m; ++j)
    for (int y = 0; y < ho; ++y)
      for (int x = 0; x < wo; ++x) {
        T best = in[((size_t)j * hi + y * ky) * wi + x * kx];
        int where = 0;
        for (int dy = 0; dy < ky; ++dy)
          for (int dx = 0; dx < kx; ++dx) {
            const T v = in[((size_t)j * hi + y * ky + dy) * wi + x * kx + dx];
            if (v > best) { best = v; where = dy * kx + dx; }
          }
        out[((size_t)j * ho + y) * wo + x] = best;
        arg[((size_t)j * ho + y) * wo + x] = (uint8_t)where;
      }
}

// Max-pooling backward (not spelled out in the paper; the derivative of a
// maximum): the gradient of a pooled value goes to the one input that won,
// every other input of the rectangle gets zero.
template <class T>
void maxpool_backward(const T* g_out, const uint8_t* arg, int m, int hi, int wi, int ky, int kx,
                      T* g_in) {
  const int ho = hi / ky, wo = wi / kx;
  std::fill(g_in, g_in + (size_t)m * hi * wi, T(0));
  for (int j = 0; j < m; ++j)
    for (int y = 0; y < ho; ++y)
      for (int x = 0; x < wo; ++x) {
        const int a = arg[((size_t)j * ho + y) * wo + x];
        const int dy = a / kx, dx = a % kx;
        g_in[((size_t)j * hi + y * ky + dy) * wi + x * kx + dx] = g_out[((size_t)j * ho + y) * wo + x];
      }
}

// Fully connected layer forward, Sec. 2.4: a_k = b_k + sum_m W[k][m] v[m].
template <class T>
void fc_forward(const T* v, int n_in, const T* bias, const T* w, int n_out, T* a) {
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (int k = 0; k < n_out; ++k) {
    T sum = bias[k];
    for (int m = 0; m < n_in; ++m) sum += w[(size_t)k * n_in + m] * v[m];
    a[k] = sum;
  }
}

// floor and ceiling of an integer quotient with a positive divisor; C's `/`
// truncates toward zero, which is wrong for the negative numerators that the
// lower bounds of Sec. 3.3 produce near the border.
inline int floor_div(int a, int b) { return (a >= 0) ? a / b : -((-a + b - 1) / b); }
inline int ceil_div(int a, int b) { return -floor_div(-a, b); }

// Back-propagation of deltas through a convolutional layer in PULL form,
// Sec. 3.3: the neuron (r, c) of input map i collects from every output map j
// that reads map i, over the rectangle of output neurons
//   max(ceil((c-Kx+1)/(Sx+1)), 0) <= x <= min(floor(c/(Sx+1)), Mx-1)
// (and the same in y), delta_j[y][x] times the weight that connected them,
// w_{j,i}[r - y(Sy+1)][c - x(Sx+1)].  The multiplication by the derivative of
// the activation is done by the caller because the layer below may be a
// max-pooling layer.
template <class T>
void conv_backward_pull(const T* delta, int ho, int wo, const T* w,
                        const std::vector<std::vector<int>>& conn, int ky, int kx, int sy, int sx,
                        int mi, int hi, int wi, T* g_in) {
  const int mo = (int)conn.size();
  std::vector<size_t> first(mo, 0);
  size_t run = 0;
  for (int j = 0; j < mo; ++j) { first[j] = run; run += conn[j].size(); }
  // transposed table (C_BP of Sec. 3.1): for input map i the (j, slot) pairs
  std::vector<std::vector<std::pair<int, size_t>>> back(mi);
  for (int j = 0; j < mo; ++j)
    for (size_t c = 0; c < conn[j].size(); ++c) back[conn[j][c]].push_back({j, first[j] + c});
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (int i = 0; i < mi; ++i)
    for (int r = 0; r < hi; ++r)
      for (int c = 0; c < wi; ++c) {
        const int ylo = std::max(ceil_div(r - ky + 1, sy + 1), 0);
        const int yhi = std::min(floor_div(r, sy + 1), ho - 1);
        const int xlo = std::max(ceil_div(c - kx + 1, sx + 1), 0);
        const int xhi = std::min(floor_div(c, sx + 1), wo - 1);
        T sum = T(0);
        for (const auto& js : back[i]) {
          const T* wk = w + js.second * (size_t)(ky * kx);
          const T* dj = delta + (size_t)js.first * ho * wo;
          for (int y = ylo; y <= yhi; ++y)
            for (int x = xlo; x <= xhi; ++x)
              sum += dj[(size_t)y * wo + x] * wk[(r - y * (sy + 1)) * kx + (c - x * (sx + 1))];
        }
        g_in[((size_t)i * hi + r) * wi + c] = sum;
      }
}

// The same quantity in PUSH form (the formulation Sec. 3.3 describes first and
// rejects for the GPU): every output delta is handed down to each input it was
// computed from.  This is the chain rule applied to conv_forward term by term;
// it exists so that the index arithmetic of the pull form has an independent
// check.
template <class T>
void conv_backward_push(const T* delta, int ho, int wo, const T* w,
                        const std::vector<std::vector<int>>& conn, int ky, int kx, int sy, int sx,
                        int mi, int hi, int wi, T* g_in) {
  std::fill(g_in, g_in + (size_t)mi * hi * wi, T(0));
  size_t slot = 0;
  for (size_t j = 0; j < conn.size(); ++j)
    for (size_t c = 0; c < conn[j].size(); ++c, ++slot) {
      const int i = conn[j][c];
      for (int y = 0; y < ho; ++y)
        for (int x = 0; x < wo; ++x)
          for (int a = 0; a < ky; ++a)
            for (int b = 0; b < kx; ++b)
              g_in[((size_t)i * hi + y * (sy + 1) + a) * wi + x * (sx + 1) + b] +=
                  delta[((size_t)j * ho + y) * wo + x] * w[slot * (size_t)(ky * kx) + a * kx + b];
    }
}

// Weight gradient of a convolutional layer (the quantity the "adjusting
// weights" kernel of Sec. 3.4 accumulates, one kernel per connection):
//   dE/dw_{j,i}[a][b] = sum_{y,x} delta_j[y][x] * in_i[y(Sy+1)+a][x(Sx+1)+b]
//   dE/db_j           = sum_{y,x} delta_j[y][x]     (one bias per output map)
template <class T>
void conv_weight_grad(const T* delta, int ho, int wo, const T* in, int hi, int wi,
                      const std::vector<std::vector<int>>& conn, int ky, int kx, int sy, int sx,
                      T* g_bias, T* g_w) {
  const int mo = (int)conn.size();
  std::vector<size_t> first(mo, 0);
  size_t run = 0;
  for (int j = 0; j < mo; ++j) { first[j] = run; run += conn[j].size(); }
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (int j = 0; j < mo; ++j) {
    T sb = T(0);
    for (int y = 0; y < ho; ++y)
      for (int x = 0; x < wo; ++x) sb += delta[((size_t)j * ho + y) * wo + x];
    g_bias[j] = sb;
    for (size_t c = 0; c < conn[j].size(); ++c) {
      const T* im = in + (size_t)conn[j][c] * hi * wi;
      for (int a = 0; a < ky; ++a)
        for (int b = 0; b < kx; ++b) {
          T s = T(0);
          for (int y = 0; y < ho; ++y)
            for (int x = 0; x < wo; ++x)
              s += delta[((size_t)j * ho + y) * wo + x] *
                   im[(size_t)(y * (sy + 1) + a) * wi + x * (sx + 1) + b];
          g_w[(first[j] + c) * (size_t)(ky * kx) + a * kx + b] = s;
        }
    }
  }
}

// Soft-max output with cross-entropy error.  The paper names neither the
// output non-linearity nor the error function; the workload definition of this
// build fixes soft-max + cross-entropy:  p = softmax(a), E = -log p[label],
// dE/da_k = p_k - [k == label].
template <class T>
T softmax_xent(const T* a, int n, int label, T* p, T* delta) {
  T mx = a[0];
  for (int k = 1; k < n; ++k) mx = std::max(mx, a[k]);
  T z = T(0);
  for (int k = 0; k < n; ++k) { p[k] = std::exp(a[k] - mx); z += p[k]; }
  for (int k = 0; k < n; ++k) p[k] /= z;
  if (delta)
    for (int k = 0; k < n; ++k) delta[k] = p[k] - (k == label ? T(1) : T(0));
  return (label >= 0 && label < n) ? -std::log(p[label]) : T(0);
}

// The output variant that follows Sec. 4 to the letter: the output neurons use the same scaled
// hyperbolic tangent as every other neuron.  The paper names no error function and no target
// coding; this variant takes the sum of squared errors against targets +1 for the image's class
// and -1 for the others (the two values the activation maps +-1 onto):
//   y_k = A tanh(B a_k),  E = 1/2 sum_k (y_k - t_k)^2,  dE/da_k = (y_k - t_k) f'(y_k).
template <class T>
T tanh_sqerr(const T* a, int n, int label, T* y, T* delta) {
  T e = T(0);
  for (int k = 0; k < n; ++k) {
    y[k] = scaled_tanh(a[k]);
    const T t = (k == label) ? T(1) : T(-1);
    e += (y[k] - t) * (y[k] - t);
    if (delta) delta[k] = (y[k] - t) * act_deriv_from_output(y[k]);
  }
  return (label >= 0 && label < n) ? e / T(2) : T(0);
}

enum OutputUnits { OUT_SOFTMAX_XENT = 0, OUT_TANH_SQERR = 1 };

// ---------------------------------------------------------------------------
// The network
// ---------------------------------------------------------------------------

struct Arch {
  std::vector<Layer> layers;  // layers[0] = network input
  int n_conv = 0;
};

bool read_int(const char*& p, int& v) {
  if (!std::isdigit((unsigned char)*p)) return false;
  long x = 0;
  while (std::isdigit((unsigned char)*p)) {
    x = x * 10 + (*p - '0');
    if (x > 1000000) return false;
    ++p;
  }
  v = (int)x;
  return true;
}

// A size: <k> (the same in both directions) or <ky>x<kx> (rows, then columns): Sec. 2.2 and 2.3 give kernels,
// skipping factors and pooling rectangles an x and a y value each.
bool read_pair(const char*& p, int& vy, int& vx) {
  if (!read_int(p, vy)) return false;
  vx = vy;
  if (*p == 'x') {
    ++p;
    if (!read_int(p, vx)) return false;
  }
  return true;
}

// Architecture string: <C>x<H>x<W> then one or more of
//   -<M>C<K>[S<s>]  convolutional layer, M maps, kernel K, skipping factor s (K, s: <k> or <ky>x<kx>)
//   -MP<K>          max-pooling over rectangles of K
//   -<N>N           fully connected layer with N neurons
// the last token being the output layer (one unit per class, Sec. 2.4).
int parse_arch(const char* s, Arch& out) {
  if (!s) return E_ARG;
  const char* p = s;
  Layer in;
  in.kind = K_INPUT;
  if (!read_int(p, in.maps) || *p++ != 'x' || !read_int(p, in.h) || *p++ != 'x' ||
      !read_int(p, in.w))
    return E_SYNTAX;
  if (in.maps < 1 || in.h < 1 || in.w < 1) return E_SHAPE;
  out.layers.clear();
  out.layers.push_back(in);
  out.n_conv = 0;
  bool seen_fc = false;
  while (*p) {
    if (*p++ != '-') return E_SYNTAX;
    const Layer& prev = out.layers.back();
    Layer l;
    if (p[0] == 'M' && p[1] == 'P') {
      p += 2;
      int ky, kx;
      if (!read_pair(p, ky, kx)) return E_SYNTAX;
      if (ky < 1 || kx < 1) return E_SHAPE;
      if (prev.kind != K_CONV) return E_SYNTAX;  // a pooling layer follows a convolutional layer (Sec. 2)
      // Sec. 2.3: pooling down-samples by exactly K; a rectangle that does not
      // tile the map is rejected rather than guessed at.
      if (prev.h % ky || prev.w % kx) return E_SHAPE;
      l.kind = K_POOL;
      l.maps = prev.maps;
      l.ky = ky;
      l.kx = kx;
      l.h = prev.h / ky;
      l.w = prev.w / kx;
    } else {
      int n;
      if (!read_int(p, n)) return E_SYNTAX;
      if (n < 1) return E_SHAPE;
      if (*p == 'C') {
        ++p;
        int ky, kx, sy = 0, sx = 0;
        if (!read_pair(p, ky, kx)) return E_SYNTAX;
        if (*p == 'S') {
          ++p;
          if (!read_pair(p, sy, sx)) return E_SYNTAX;
        }
        if (ky < 1 || kx < 1) return E_SHAPE;
        if (seen_fc) return E_SYNTAX;
        l.kind = K_CONV;
        l.maps = n;
        l.ky = ky;
        l.kx = kx;
        l.sy = sy;
        l.sx = sx;
        l.h = conv_out_size(prev.h, ky, sy);
        l.w = conv_out_size(prev.w, kx, sx);
        if (l.h < 1 || l.w < 1) return E_SHAPE;
        l.conn.assign(n, {});
        for (int j = 0; j < n; ++j)
          for (int i = 0; i < prev.maps; ++i) l.conn[j].push_back(i);
        ++out.n_conv;
      } else if (*p == 'N') {
        ++p;
        l.kind = K_FC;
        l.maps = n;
        l.h = l.w = 1;
        seen_fc = true;
      } else {
        return E_SYNTAX;
      }
    }
    out.layers.push_back(l);
  }
  if (out.layers.size() < 2 || out.layers.back().kind != K_FC) return E_SYNTAX;
  return E_OK;
}

template <class T>
struct Net {
  Arch arch;
  std::vector<T> weights;  // canonical layout, see layout()
  // optional fixed image-processing layer (Sec. 2.1): n filters of fe_k x fe_k,
  // filter f reads raw channel fe_src[f]; valid correlation, no bias, linear,
  // never trained, no delta computed into it.
  int fe_n = 0, fe_k = 0, fe_c = 0;
  std::vector<T> fe_filt;
  std::vector<int> fe_src;

  std::vector<std::vector<T>> act;     // output of every layer (layer 0 = net input)
  std::vector<std::vector<T>> gout;    // dE/d(output) of every layer >= 1
  std::vector<std::vector<T>> delta;   // dE/d(pre-activation), conv and FC layers
  std::vector<std::vector<uint8_t>> arg;
  std::vector<T> grad;                 // canonical layout
  T loss = T(0);
  int out_units = OUT_SOFTMAX_XENT;    // what the last layer computes and which error it is trained on

  std::vector<Layer>& L() { return arch.layers; }
  int n_layers() const { return (int)arch.layers.size(); }
  int fc_inputs(int l) const {
    const Layer& p = arch.layers[l - 1];
    return p.maps * p.h * p.w;
  }

  // Canonical weight layout: layer by layer; conv: bias[M] then one K*K block
  // per connection, output map ascending, connected input map ascending inside
  // it; FC: bias[N] then W[N][n_in] row-major with n_in index (map*H + y)*W + x.
  void layout() {
    size_t off = 0;
    for (int l = 1; l < n_layers(); ++l) {
      Layer& a = L()[l];
      a.b_off = off;
      a.n_weights = 0;
      if (a.kind == K_CONV) {
        size_t nc = 0;
        for (auto& r : a.conn) nc += r.size();
        a.w_off = off + a.maps;
        a.n_weights = a.maps + nc * a.ky * a.kx;
      } else if (a.kind == K_FC) {
        a.w_off = off + a.maps;
        a.n_weights = (size_t)a.maps * (1 + fc_inputs(l));
      }
      off += a.n_weights;
    }
    weights.assign(off, T(0));
    grad.assign(off, T(0));
    act.assign(n_layers(), {});
    gout.assign(n_layers(), {});
    delta.assign(n_layers(), {});
    arg.assign(n_layers(), {});
    for (int l = 0; l < n_layers(); ++l) {
      const size_t n = (size_t)L()[l].maps * L()[l].h * L()[l].w;
      act[l].assign(n, T(0));
      gout[l].assign(n, T(0));
      if (L()[l].kind == K_CONV || L()[l].kind == K_FC) delta[l].assign(n, T(0));
      if (L()[l].kind == K_POOL) arg[l].assign(n, 0);
    }
  }

  size_t raw_image_size() const {
    const Layer& in = arch.layers[0];
    if (fe_n) return (size_t)fe_c * (in.h + fe_k - 1) * (in.w + fe_k - 1);
    return (size_t)in.maps * in.h * in.w;
  }

  // Forward pass: Sec. 2.1 (fixed filters), 2.2, 2.3, 2.4 in network order.
  void forward(const float* image) {
    Layer& in = L()[0];
    if (fe_n) {
      const int rh = in.h + fe_k - 1, rw = in.w + fe_k - 1;
      std::vector<T> raw(raw_image_size());
      for (size_t t = 0; t < raw.size(); ++t) raw[t] = (T)image[t];
      for (int f = 0; f < fe_n; ++f) {
        std::vector<std::vector<int>> one(1, std::vector<int>(1, fe_src[f]));
        conv_forward<T>(raw.data(), fe_c, rh, rw, nullptr, fe_filt.data() + (size_t)f * fe_k * fe_k,
                        one, fe_k, fe_k, 0, 0, in.h, in.w, false,
                        act[0].data() + (size_t)f * in.h * in.w);
      }
    } else {
      for (size_t t = 0; t < act[0].size(); ++t) act[0][t] = (T)image[t];
    }
    forward_from(1);
  }

  // Layers first .. top, the input of layer `first` being current.
  void forward_from(int first) {
    for (int l = first; l < n_layers(); ++l) {
      Layer& a = L()[l];
      const Layer& p = L()[l - 1];
      if (a.kind == K_CONV) {
        conv_forward<T>(act[l - 1].data(), p.maps, p.h, p.w, &weights[a.b_off], &weights[a.w_off],
                        a.conn, a.ky, a.kx, a.sy, a.sx, a.h, a.w, true, act[l].data());
      } else if (a.kind == K_POOL) {
        maxpool_forward<T>(act[l - 1].data(), p.maps, p.h, p.w, a.ky, a.kx, act[l].data(),
                           arg[l].data());
      } else {
        fc_forward<T>(act[l - 1].data(), fc_inputs(l), &weights[a.b_off], &weights[a.w_off], a.maps,
                      act[l].data());
        if (l + 1 < n_layers()) {
          for (auto& v : act[l]) v = scaled_tanh(v);  // hidden units: scaled tanh (Sec. 4)
        } else if (out_units == OUT_TANH_SQERR) {
          for (auto& v : act[l]) v = scaled_tanh(v);
        } else {
          std::vector<T> logits(act[l]);
          softmax_xent<T>(logits.data(), a.maps, -1, act[l].data(), nullptr);
        }
      }
    }
  }

  // E of the last forward pass for `label`; when d is given, also dE/d(pre-activation) of the
  // output neurons.  Soft-max: act[top] holds the probabilities, delta_k = p_k - [k == label].
  // Scaled tanh: act[top] holds the outputs, delta_k = (y_k - t_k) f'(y_k), t = +-1.
  T error_and_output_delta(int label, T* d) {
    const int top = n_layers() - 1;
    const int n = L()[top].maps;
    const std::vector<T>& y = act[top];
    if (out_units == OUT_TANH_SQERR) {
      T e = T(0);
      for (int k = 0; k < n; ++k) {
        const T t = (k == label) ? T(1) : T(-1);
        e += (y[k] - t) * (y[k] - t);
        if (d) d[k] = (y[k] - t) * act_deriv_from_output(y[k]);
      }
      return e / T(2);
    }
    if (d)
      for (int k = 0; k < n; ++k) d[k] = y[k] - (k == label ? T(1) : T(0));
    return -std::log(y[label]);
  }

  // Backward pass and gradients with every weight still at its pre-update
  // value (Sec. 3.3 for the deltas, Sec. 3.4 for the weight gradients).
  // Requires forward() on the same image.  Nothing is propagated into the
  // network input: there is nothing to adjust below it.
  void backward(int label) {
    const int top = n_layers() - 1;
    loss = error_and_output_delta(label, delta[top].data());
    for (int l = top; l >= 1; --l) {
      Layer& a = L()[l];
      const Layer& p = L()[l - 1];
      if (a.kind == K_FC) {
        const int n_in = fc_inputs(l);
        if (l < top)
          for (size_t t = 0; t < delta[l].size(); ++t)
            delta[l][t] = gout[l][t] * act_deriv_from_output(act[l][t]);
        // gradients of this layer: dE/dW[k][m] = delta_k v_m, dE/db_k = delta_k
        for (int k = 0; k < a.maps; ++k) {
          grad[a.b_off + k] = delta[l][k];
          for (int m = 0; m < n_in; ++m)
            grad[a.w_off + (size_t)k * n_in + m] = delta[l][k] * act[l - 1][m];
        }
        if (l - 1 >= 1)
          for (int m = 0; m < n_in; ++m) {
            T s = T(0);
            for (int k = 0; k < a.maps; ++k) s += weights[a.w_off + (size_t)k * n_in + m] * delta[l][k];
            gout[l - 1][m] = s;
          }
      } else if (a.kind == K_POOL) {
        maxpool_backward<T>(gout[l].data(), arg[l].data(), p.maps, p.h, p.w, a.ky, a.kx,
                            gout[l - 1].data());
      } else {  // K_CONV
        // the summed error is multiplied by the activation function's derivative (Sec. 3.3)
        for (size_t t = 0; t < delta[l].size(); ++t)
          delta[l][t] = gout[l][t] * act_deriv_from_output(act[l][t]);
        conv_weight_grad<T>(delta[l].data(), a.h, a.w, act[l - 1].data(), p.h, p.w, a.conn, a.ky,
                            a.kx, a.sy, a.sx, &grad[a.b_off], &grad[a.w_off]);
        if (l - 1 >= 1)
          conv_backward_pull<T>(delta[l].data(), a.h, a.w, &weights[a.w_off], a.conn, a.ky, a.kx,
                                a.sy, a.sx, p.maps, p.h, p.w, gout[l - 1].data());
      }
    }
  }

  // One step of on-line gradient descent (Sec. 1, Sec. 4: the weights are
  // adjusted after each image): w <- w - lr * dE/dw.  Plain SGD; the paper
  // mentions neither momentum nor weight decay.
  T train_step(const float* image, int label, T lr) {
    forward(image);
    backward(label);
    for (size_t t = 0; t < weights.size(); ++t) weights[t] -= lr * grad[t];
    return loss;
  }
};

// Tie-break hints for a max-pooling layer (test support).  Two implementations that sum in
// different orders can disagree on the winner of a rectangle only where its two best values are
// nearly equal; there both choices are valid results.  A hinted winner is adopted where the
// oracle's own maximum exceeds the hinted value by at most tol * max|input|, and refused
// otherwise.  After an adoption the layers above are recomputed from the changed pooled values.
template <class T>
int adopt_argmax_hint(Net<T>& n, int layer, const uint8_t* hint, double tol, int* adopted, int* rejected) {
  if (layer < 1 || layer >= n.n_layers() || n.L()[layer].kind != K_POOL) return E_ARG;
  const Layer& a = n.L()[layer];
  const Layer& p = n.L()[layer - 1];
  double scale = 0;
  for (const T& v : n.act[layer - 1]) scale = std::max(scale, (double)std::fabs(v));
  int na = 0, nr = 0;
  for (int j = 0; j < a.maps; ++j)
    for (int y = 0; y < a.h; ++y)
      for (int x = 0; x < a.w; ++x) {
        const size_t o = ((size_t)j * a.h + y) * a.w + x;
        const int h = hint[o];
        if (h == n.arg[layer][o]) continue;
        if (h >= a.ky * a.kx) { ++nr; continue; }
        const T vh = n.act[layer - 1][((size_t)j * p.h + y * a.ky + h / a.kx) * p.w + x * a.kx + h % a.kx];
        if ((double)(n.act[layer][o] - vh) <= tol * scale) {
          n.arg[layer][o] = (uint8_t)h;
          n.act[layer][o] = vh;
          ++na;
        } else {
          ++nr;
        }
      }
  if (na && layer + 1 < n.n_layers()) n.forward_from(layer + 1);
  if (adopted) *adopted = na;
  if (rejected) *rejected = nr;
  return E_OK;
}

struct Handle {
  int precision;  // 32 or 64
  Net<double>* d = nullptr;
  Net<float>* f = nullptr;
  ~Handle() { delete d; delete f; }
};

template <class T>
int set_table(Net<T>& n, int conv_index, const uint8_t* table) {
  int seen = 0;
  for (int l = 1; l < n.n_layers(); ++l) {
    Layer& a = n.L()[l];
    if (a.kind != K_CONV) continue;
    if (seen++ != conv_index) continue;
    const int mi = n.L()[l - 1].maps;
    std::vector<std::vector<int>> conn(a.maps);
    for (int j = 0; j < a.maps; ++j) {
      for (int i = 0; i < mi; ++i)
        if (table[(size_t)j * mi + i]) conn[j].push_back(i);
      if (conn[j].empty()) return E_ARG;  // an output map with no input is not a layer of Sec. 2.2
    }
    a.conn = conn;
    n.layout();
    return E_OK;
  }
  return E_ARG;
}

template <class T>
int set_frontend(Net<T>& n, int n_filters, int k, int n_src, const float* filt, const int32_t* src) {
  if (n_filters != n.L()[0].maps || k < 1 || n_src < 1 || !filt || !src) return E_ARG;
  for (int f = 0; f < n_filters; ++f)
    if (src[f] < 0 || src[f] >= n_src) return E_ARG;
  n.fe_n = n_filters;
  n.fe_k = k;
  n.fe_c = n_src;
  n.fe_filt.assign((size_t)n_filters * k * k, T(0));
  for (size_t t = 0; t < n.fe_filt.size(); ++t) n.fe_filt[t] = (T)filt[t];
  n.fe_src.assign(src, src + n_filters);
  return E_OK;
}

}  // namespace

#define WITH_NET(h, expr)                 \
  do {                                    \
    if ((h)->precision == 64) {           \
      auto& net = *(h)->d;                \
      expr;                               \
    } else {                              \
      auto& net = *(h)->f;                \
      expr;                               \
    }                                     \
  } while (0)

extern "C" {

typedef struct Handle oracle_t;

int oracle_conv_out_size(int m_prev, int k, int s) { return conv_out_size(m_prev, k, s); }

int oracle_create(const char* arch, int precision, oracle_t** out) {
  if (!out || (precision != 32 && precision != 64)) return E_ARG;
  Arch a;
  int rc = parse_arch(arch, a);
  if (rc) return rc;
  Handle* h = new Handle;
  h->precision = precision;
  if (precision == 64) { h->d = new Net<double>; h->d->arch = a; h->d->layout(); }
  else { h->f = new Net<float>; h->f->arch = a; h->f->layout(); }
  *out = h;
  return E_OK;
}

void oracle_destroy(oracle_t* h) { delete h; }

int oracle_set_connection_table(oracle_t* h, int conv_index, const uint8_t* table) {
  if (!h || !table) return E_ARG;
  int rc;
  WITH_NET(h, rc = set_table(net, conv_index, table));
  return rc;
}

int oracle_set_fixed_frontend(oracle_t* h, int n_filters, int k, int n_src_channels,
                              const float* filters, const int32_t* src_channel) {
  if (!h) return E_ARG;
  int rc;
  WITH_NET(h, rc = set_frontend(net, n_filters, k, n_src_channels, filters, src_channel));
  return rc;
}

// 0: soft-max outputs trained on the cross-entropy error (default); 1: scaled-tanh outputs trained
// on the squared error against +-1 targets.
int oracle_set_output_units(oracle_t* h, int kind) {
  if (!h || (kind != OUT_SOFTMAX_XENT && kind != OUT_TANH_SQERR)) return E_ARG;
  WITH_NET(h, net.out_units = kind);
  return E_OK;
}

size_t oracle_num_weights(oracle_t* h) {
  size_t n;
  WITH_NET(h, n = net.weights.size());
  return n;
}

int oracle_num_layers(oracle_t* h) {
  int n;
  WITH_NET(h, n = net.n_layers());
  return n;
}

// info = {kind, maps, h, w, Ky, Sy, Kx, Sx}
int oracle_layer_info(oracle_t* h, int layer, int32_t* info) {
  if (!h || !info) return E_ARG;
  int rc = E_OK;
  WITH_NET(h, {
    if (layer < 0 || layer >= net.n_layers()) rc = E_ARG;
    else {
      const Layer& a = net.L()[layer];
      info[0] = a.kind; info[1] = a.maps; info[2] = a.h; info[3] = a.w; info[4] = a.ky; info[5] = a.sy;
      info[6] = a.kx; info[7] = a.sx;
    }
  });
  return rc;
}

size_t oracle_image_size(oracle_t* h) {
  size_t n;
  WITH_NET(h, n = net.raw_image_size());
  return n;
}

int oracle_set_weights(oracle_t* h, const double* src, size_t n) {
  if (!h || !src) return E_ARG;
  int rc = E_OK;
  WITH_NET(h, {
    if (n != net.weights.size()) rc = E_ARG;
    else for (size_t t = 0; t < n; ++t) net.weights[t] = (decltype(net.loss))src[t];
  });
  return rc;
}

int oracle_get_weights(oracle_t* h, double* dst, size_t n) {
  if (!h || !dst) return E_ARG;
  int rc = E_OK;
  WITH_NET(h, {
    if (n != net.weights.size()) rc = E_ARG;
    else for (size_t t = 0; t < n; ++t) dst[t] = (double)net.weights[t];
  });
  return rc;
}

int oracle_forward(oracle_t* h, const float* image, double* probs) {
  if (!h || !image) return E_ARG;
  WITH_NET(h, {
    net.forward(image);
    if (probs) for (size_t t = 0; t < net.act.back().size(); ++t) probs[t] = (double)net.act.back()[t];
  });
  return E_OK;
}

static int check_label(oracle_t* h, int label) {
  int n;
  WITH_NET(h, n = net.L().back().maps);
  return (label >= 0 && label < n) ? E_OK : E_ARG;
}

int oracle_train_step(oracle_t* h, const float* image, int32_t label, double lr, double* loss) {
  if (!h || !image) return E_ARG;
  if (check_label(h, label)) return E_ARG;
  WITH_NET(h, {
    auto e = net.train_step(image, label, (decltype(net.loss))lr);
    if (loss) *loss = (double)e;
  });
  return E_OK;
}

// Forward state must be current (oracle_forward, possibly followed by oracle_adopt_argmax_hint):
// backward pass, gradients and the SGD update of one on-line step.
int oracle_backward_update(oracle_t* h, int32_t label, double lr, double* loss) {
  if (!h) return E_ARG;
  if (check_label(h, label)) return E_ARG;
  WITH_NET(h, {
    net.backward(label);
    for (size_t t = 0; t < net.weights.size(); ++t) net.weights[t] -= (decltype(net.loss))lr * net.grad[t];
    if (loss) *loss = (double)net.loss;
  });
  return E_OK;
}

int oracle_adopt_argmax_hint(oracle_t* h, int layer, const uint8_t* hint, double tol, int* adopted,
                             int* rejected) {
  if (!h || !hint) return E_ARG;
  int rc;
  WITH_NET(h, rc = adopt_argmax_hint(net, layer, hint, tol, adopted, rejected));
  return rc;
}

int oracle_train_many(oracle_t* h, const float* images, const int32_t* labels, size_t n, double lr) {
  if (!h || !images || !labels) return E_ARG;
  size_t sz = oracle_image_size(h);
  for (size_t t = 0; t < n; ++t) {
    int rc = oracle_train_step(h, images + t * sz, labels[t], lr, nullptr);
    if (rc) return rc;
  }
  return E_OK;
}

int oracle_forward_many(oracle_t* h, const float* images, size_t n, double* probs) {
  if (!h || !images) return E_ARG;
  size_t sz = oracle_image_size(h);
  size_t nc;
  WITH_NET(h, nc = net.act.back().size());
  for (size_t t = 0; t < n; ++t) oracle_forward(h, images + t * sz, probs ? probs + t * nc : nullptr);
  return E_OK;
}

// Gradient of E for (image, label) at the current weights, canonical layout; no update.
int oracle_gradients(oracle_t* h, const float* image, int32_t label, double* grad, double* loss) {
  if (!h || !image) return E_ARG;
  if (check_label(h, label)) return E_ARG;
  WITH_NET(h, {
    net.forward(image);
    net.backward(label);
    if (grad) for (size_t t = 0; t < net.grad.size(); ++t) grad[t] = (double)net.grad[t];
    if (loss) *loss = (double)net.loss;
  });
  return E_OK;
}

// E for (image, label) at the current weights (for finite differences).
int oracle_loss(oracle_t* h, const float* image, int32_t label, double* loss) {
  if (!h || !image || !loss) return E_ARG;
  if (check_label(h, label)) return E_ARG;
  WITH_NET(h, {
    net.forward(image);
    *loss = (double)net.error_and_output_delta(label, nullptr);
  });
  return E_OK;
}

int oracle_get_activation(oracle_t* h, int layer, double* dst) {
  if (!h || !dst) return E_ARG;
  int rc = E_OK;
  WITH_NET(h, {
    if (layer < 0 || layer >= net.n_layers()) rc = E_ARG;
    else for (size_t t = 0; t < net.act[layer].size(); ++t) dst[t] = (double)net.act[layer][t];
  });
  return rc;
}

// dE/d(pre-activation) of a convolutional or fully connected layer, dense.
int oracle_get_delta(oracle_t* h, int layer, double* dst) {
  if (!h || !dst) return E_ARG;
  int rc = E_OK;
  WITH_NET(h, {
    if (layer < 1 || layer >= net.n_layers() || net.delta[layer].empty()) rc = E_ARG;
    else for (size_t t = 0; t < net.delta[layer].size(); ++t) dst[t] = (double)net.delta[layer][t];
  });
  return rc;
}

int oracle_get_argmax(oracle_t* h, int layer, uint8_t* dst) {
  if (!h || !dst) return E_ARG;
  int rc = E_OK;
  WITH_NET(h, {
    if (layer < 1 || layer >= net.n_layers() || net.arg[layer].empty()) rc = E_ARG;
    else std::memcpy(dst, net.arg[layer].data(), net.arg[layer].size());
  });
  return rc;
}

// ---- single-operation entry points (double), for the pins and for
// ---- layer-isolated parity checks.  table is [mo][mi] of 0/1.

static std::vector<std::vector<int>> table_to_conn(const uint8_t* table, int mo, int mi) {
  std::vector<std::vector<int>> conn(mo);
  for (int j = 0; j < mo; ++j)
    for (int i = 0; i < mi; ++i)
      if (!table || table[(size_t)j * mi + i]) conn[j].push_back(i);
  return conn;
}

int oracle_op_conv_forward(const double* in, int mi, int hi, int wi, const double* bias,
                           const double* w, const uint8_t* table, int mo, int ky, int kx, int sy,
                           int sx, int apply_act, double* out) {
  const int ho = conv_out_size(hi, ky, sy), wo = conv_out_size(wi, kx, sx);
  if (ho < 1 || wo < 1) return E_SHAPE;
  conv_forward<double>(in, mi, hi, wi, bias, w, table_to_conn(table, mo, mi), ky, kx, sy, sx, ho, wo,
                       apply_act != 0, out);
  return E_OK;
}

int oracle_op_maxpool_forward(const double* in, int m, int hi, int wi, int ky, int kx, double* out,
                              uint8_t* arg) {
  if (ky < 1 || kx < 1 || hi % ky || wi % kx) return E_SHAPE;
  maxpool_forward<double>(in, m, hi, wi, ky, kx, out, arg);
  return E_OK;
}

int oracle_op_maxpool_backward(const double* g_out, const uint8_t* arg, int m, int hi, int wi, int ky,
                               int kx, double* g_in) {
  if (ky < 1 || kx < 1 || hi % ky || wi % kx) return E_SHAPE;
  maxpool_backward<double>(g_out, arg, m, hi, wi, ky, kx, g_in);
  return E_OK;
}

int oracle_op_conv_backward(const double* delta, const double* w, const uint8_t* table, int mo, int mi,
                            int hi, int wi, int ky, int kx, int sy, int sx, int push, double* g_in) {
  const int ho = conv_out_size(hi, ky, sy), wo = conv_out_size(wi, kx, sx);
  if (ho < 1 || wo < 1) return E_SHAPE;
  auto conn = table_to_conn(table, mo, mi);
  if (push) conv_backward_push<double>(delta, ho, wo, w, conn, ky, kx, sy, sx, mi, hi, wi, g_in);
  else conv_backward_pull<double>(delta, ho, wo, w, conn, ky, kx, sy, sx, mi, hi, wi, g_in);
  return E_OK;
}

int oracle_op_conv_weight_grad(const double* delta, const double* in, const uint8_t* table, int mo,
                               int mi, int hi, int wi, int ky, int kx, int sy, int sx, double* g_bias,
                               double* g_w) {
  const int ho = conv_out_size(hi, ky, sy), wo = conv_out_size(wi, kx, sx);
  if (ho < 1 || wo < 1) return E_SHAPE;
  conv_weight_grad<double>(delta, ho, wo, in, hi, wi, table_to_conn(table, mo, mi), ky, kx, sy, sx,
                           g_bias, g_w);
  return E_OK;
}

int oracle_op_fc_forward(const double* v, int n_in, const double* bias, const double* w, int n_out,
                         double* a) {
  fc_forward<double>(v, n_in, bias, w, n_out, a);
  return E_OK;
}

double oracle_op_act(double a) { return scaled_tanh<double>(a); }
double oracle_op_act_deriv_from_output(double y) { return act_deriv_from_output<double>(y); }

double oracle_op_softmax_xent(const double* a, int n, int label, double* p, double* delta) {
  return softmax_xent<double>(a, n, label, p, delta);
}

double oracle_op_tanh_sqerr(const double* a, int n, int label, double* y, double* delta) {
  return tanh_sqerr<double>(a, n, label, y, delta);
}

int oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
  return omp_get_max_threads();
#else
  (void)n;
  return 1;
#endif
}

}  // extern "C"
