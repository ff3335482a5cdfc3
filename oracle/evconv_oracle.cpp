// CPU oracle for incremental CNN inference on event-camera inputs (Ev-Conv).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the HIP library is
// checked against; only tests, the smoke check and the benchmark's cpu_baseline leg may load
// it.  It shares no code, header, table or helper with the HIP path and never calls it.
//
// Two independent halves that must agree (Eq.2 of the paper, the telescoping sum
// y(n) = y(n-m) + sum of increments):
//   * dense_forward(): the plain definition - a regular forward pass of the whole network on a
//     full input tensor (textbook convolution, ReLU, sigmoid, max-pool, bilinear x2, mean).
//     "Refresh" (Drift Errors section) is exactly this pass, storing every accumulated tensor.
//   * step(): the incremental algorithm in the paper's order: input increment (Eq.1), then per
//     layer the increment operator of "Implementation of Increment Layers": linear ops on the
//     increment alone (Eq.9-10), addition with OR-ed masks (Eq.11), activation through the
//     accumulated input x_acc (Eq.12-14), and the output sum (Eq.2).
//
// Arithmetic is templated: T = double (reference state) or T = float (every operation in
// binary32, used for bit-exact checks of elementwise kernels and for the drift study).  The
// input increment itself is always one binary32 subtraction (Eq.1 on fp32 frames).
//
// Readings where the paper is silent (all mirrored in the project's design notes):
//   * mask = per-site "any channel nonzero" set; a tile bitmap/occupancy word is derived from
//     it for a given tile size and never influences a value (a mask may only skip zeros).
//   * zero test is `!= 0` on the stored value: -0 is inactive, denormals and NaN are active.
//   * after an activation / conv / max-pool the active set is value-pruned (sites whose output
//     increment is zero in every channel are dropped); the un-pruned "touched" set (the paper's
//     Eq.13 mask y_m = x_m pushed through the operator's footprint) is kept beside it.
//     Bare add, concat, upsample and mean-pool keep the structural set (Eq.11b: OR).
//   * bias enters only in the dense pass (the increment of a constant is zero).
//   * padding is zero padding; max-pool pads with -inf; bilinear x2 uses half-pixel centres
//     with clamped borders (weights 0.25 / 0.75).
//   * a linear op without activation emits y_inc = theta_L(x_inc) itself (Eq.10), not the
//     difference of the accumulated sums.
//   * sparsification layer (Eq.3-8; the printed Eq.4 and Eq.8 disagree in sign and Eq.8 counts
//     the old residual twice): delta(-1) = 0; x_corr = delta(n-1) + x_inc(n);
//     y_inc = k * floor(0.5 + x_corr / k); delta(n) = x_corr - y_inc, applied to the elements
//     whose x_inc is nonzero (for the others the same formulas give y_inc = 0).  This keeps
//     sum(y_inc) + delta == sum(x_inc) and -k/2 <= delta < k/2, which is what the text asks of
//     the residual.  A refresh is a regular forward pass (the layer is the identity) and clears
//     delta.  k = t_p * RMS(layer input at the last refresh), rounded to 8 fraction bits so
//     that both sides of a comparison use the identical step (the paper says "t_p times the L2
//     norm of a rolling average of the input" without giving window or normalisation);
//     k == 0 makes the layer the identity.
//   * recurrence (the paper's evaluation networks are recurrent, "Experiments"; how a recurrent
//     state is carried is not said): a DELAY node stands for "the value of a later node X at the
//     previous step".  Its increment at step n is X's increment of step n-1, its mask X's mask
//     of step n-1 (the state is one more input whose change is known); the state before the first
//     frame is zero, so after a reset the first step's increment of the DELAY node is X's whole
//     value, at every site.  A regular forward pass in mid-stream (refresh) keeps the recurrent
//     state: the DELAY node then holds X's value of the previous step.
//   * elementwise multiply (Eq.15-17) keeps the accumulated values of both inputs; the output
//     increment uses the accumulators as they were before this step, then both are advanced;
//     its mask is the OR of the input masks (Eq.16, structural, like addition).
//
// Parity pins live in tests/ (CPU, "not gpu"): dense ops against PyTorch CPU fp64 routines,
// Eq.2 invariant against the dense pass, linearity, zero increment, tile independence,
// refresh equivalence, brute-force lists with exact integer arithmetic, closed-form touched
// sets for a single active pixel.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

namespace {

enum Op { OP_CONV = 0, OP_ADD, OP_CONCAT, OP_UP2X, OP_MAXPOOL, OP_GAP, OP_LINEAR, OP_ACT, OP_SPARSIFY, OP_MUL,
          OP_DELAY };  // OP_DELAY: in0 = the later node X it delays, in1 = an earlier node (or -1) with its height and width
enum Act { ACT_NONE = 0, ACT_RELU, ACT_SIGMOID, ACT_TANH, ACT_ONE_MINUS };  // ONE_MINUS: 1 - z

struct NodeDesc {
  int op, act, in0, in1, c_in, c_out, k, stride, pad;
  long long w_off, b_off;
  int is_output;
};
constexpr int kDescInts = 12;  // ints per node in the marshalled description

template <class T>
T activate(int act, T v) {
  if (act == ACT_RELU) return v > T(0) ? v : T(0);
  if (act == ACT_SIGMOID) return T(1) / (T(1) + std::exp(-v));
  if (act == ACT_TANH) return std::tanh(v);
  if (act == ACT_ONE_MINUS) return T(1) - v;
  return v;
}

struct Shape {
  int c = 0, h = 0, w = 0;
  size_t sites() const { return size_t(h) * w; }
  size_t elems() const { return sites() * c; }
};

// bilinear x2, half-pixel centres: output index o reads source i0 (weight w0) and i1 (w1)
inline void up2_src(int o, int n_in, int& i0, int& i1, double& w0, double& w1) {
  int i = o >> 1;
  if ((o & 1) == 0) { i0 = std::max(i - 1, 0); i1 = i; w0 = 0.25; w1 = 0.75; }
  else { i0 = i; i1 = std::min(i + 1, n_in - 1); w0 = 0.75; w1 = 0.25; }
}

template <class T>
struct NodeState {
  Shape shp;                     // output shape
  std::vector<T> z;              // accumulated pre-activation / accumulated linear result
  std::vector<T> z2;             // elementwise multiply: accumulated second input (z: the first)
  std::vector<T> pool_in;        // max-pool: accumulated input (input shape)
  std::vector<T> dy;             // this step's output increment, HWC, zero off the active set
  std::vector<uint8_t> active;   // value-pruned (or structural) active set S
  std::vector<uint8_t> touched;  // structural touched set T
  std::vector<T> y;              // output nodes: running sum of increments (Eq.2)
  std::vector<T> dz, da;         // dense pass: pre-activation and value of this node
  float k = 0.f;                 // sparsification layer: rounding step (z holds the residual delta)
  float k_fixed = -1.f;          // >= 0: step given by the description instead of t_p * RMS
  bool keeps_z = false, structural = false;
  // multiply-accumulate counters of a conv / linear node (the paper's "MFLOPs" columns, Tables I-III,
  // under an explicit counting rule; one MAC = one weight times one input element):
  //   macs_site          executed by the last step when only nonzero work is done: over the touched
  //                      outputs, the (tap, output) pairs whose input site is inside the image and
  //                      active, times c_in * c_out
  //   macs_dense         a regular forward pass: the pairs whose input site is inside the image
  //                      (zero padding costs nothing), times c_in * c_out
  //   macs_dense_nominal outputs * k * k * c_in * c_out (padding counted: the usual quoted figure)
  double macs_site = 0, macs_dense = 0, macs_dense_nominal = 0;
};

template <class T>
struct Net {
  std::vector<NodeDesc> nodes;
  std::vector<double> weights;
  Shape in;
  std::vector<float> x_prev;          // CHW, the cached previous frame
  std::vector<T> dx;                  // HWC input increment
  std::vector<uint8_t> s0;            // input active set
  std::vector<T> x_dense;             // HWC copy of the frame for the dense pass
  std::vector<NodeState<T>> st;
  bool has_state = false;
  bool last_dense = true;   // the previous pass was a regular forward pass (DELAY nodes)
  bool first_pass = true;   // inside reset(): the recurrent state is zero
  double sparsify_tp = 0.0;

  const Shape& shape_of(int i) const { return i < 0 ? in : st[i].shp; }
  const std::vector<T>& dy_of(int i) const { return i < 0 ? dx : st[i].dy; }
  const std::vector<uint8_t>& set_of(int i) const { return i < 0 ? s0 : st[i].active; }
  const std::vector<T>& dense_of(int i) const { return i < 0 ? x_dense : st[i].da; }

  // weights of conv/linear node i, re-laid as [ky][kx][ci][co] so that the innermost (output
  // channel) loop of the contraction walks contiguous memory; row() is the c_out-vector of
  // W[:, ci, ky, kx]
  std::vector<std::vector<T>> w_taps;
  inline const T* row(int i, const NodeDesc& nd, int ci, int ky, int kx) const {
    return &w_taps[i][((size_t(ky) * nd.k + kx) * nd.c_in + ci) * nd.c_out];
  }

  int init(int n_nodes, const int* desc, const double* w, long long n_w, int c, int h, int wd) {
    in.c = c; in.h = h; in.w = wd;
    weights.assign(w, w + n_w);
    nodes.resize(n_nodes);
    st.resize(n_nodes);
    w_taps.resize(n_nodes);
    for (int i = 0; i < n_nodes; ++i) {
      const int* d = desc + size_t(i) * kDescInts;
      NodeDesc& nd = nodes[i];
      nd.op = d[0]; nd.act = d[1]; nd.in0 = d[2]; nd.in1 = d[3]; nd.c_in = d[4]; nd.c_out = d[5];
      nd.k = d[6]; nd.stride = d[7]; nd.pad = d[8]; nd.w_off = d[9]; nd.b_off = d[10];
      nd.is_output = d[11];
      if (nd.op == OP_DELAY) {
        if (nd.in0 <= i || nd.in0 >= n_nodes || nd.in1 >= i || nd.in1 < -1 || nd.act != ACT_NONE) return 1;
      } else if (nd.in0 >= i || nd.in1 >= i || nd.in0 < -1) {
        return 1;
      }
      Shape a = shape_of(nd.op == OP_DELAY ? nd.in1 : nd.in0), o;
      switch (nd.op) {
        case OP_CONV:
          if (a.c != nd.c_in) return 2;
          o.c = nd.c_out;
          o.h = (a.h + 2 * nd.pad - nd.k) / nd.stride + 1;
          o.w = (a.w + 2 * nd.pad - nd.k) / nd.stride + 1;
          break;
        case OP_MAXPOOL:
          if (nd.act != ACT_NONE) return 3;
          o.c = a.c;
          o.h = (a.h + 2 * nd.pad - nd.k) / nd.stride + 1;
          o.w = (a.w + 2 * nd.pad - nd.k) / nd.stride + 1;
          break;
        case OP_ADD: {
          Shape b = shape_of(nd.in1);
          if (b.c != a.c || b.h != a.h || b.w != a.w) return 4;
          o = a;
          break;
        }
        case OP_MUL: {
          Shape b = shape_of(nd.in1);
          if (b.c != a.c || b.h != a.h || b.w != a.w) return 4;
          if (nd.act != ACT_NONE) return 3;
          o = a;
          break;
        }
        case OP_ACT: o = a; break;
        case OP_SPARSIFY:
          if (nd.act != ACT_NONE) return 3;
          o = a;
          if (nd.w_off >= 0) {
            if (nd.w_off >= n_w) return 9;
            st[i].k_fixed = float(weights[nd.w_off]);
          }
          break;
        case OP_CONCAT: {
          Shape b = shape_of(nd.in1);
          if (b.h != a.h || b.w != a.w) return 5;
          o = a; o.c = a.c + b.c;
          break;
        }
        case OP_UP2X: o.c = a.c; o.h = 2 * a.h; o.w = 2 * a.w; break;
        case OP_GAP: o.c = a.c; o.h = 1; o.w = 1; break;
        case OP_DELAY: o.c = nd.c_out; o.h = a.h; o.w = a.w; break;  // checked against X's shape below
        case OP_LINEAR:
          if (a.h != 1 || a.w != 1 || a.c != nd.c_in) return 6;
          o.c = nd.c_out; o.h = 1; o.w = 1;
          break;
        default: return 7;
      }
      if (o.h <= 0 || o.w <= 0) return 8;
      NodeState<T>& s = st[i];
      s.shp = o;
      s.keeps_z = (nd.op == OP_CONV || nd.op == OP_LINEAR || nd.op == OP_GAP || nd.op == OP_ACT ||
                   nd.op == OP_SPARSIFY || nd.act != ACT_NONE) && nd.op != OP_MAXPOOL;
      s.structural = (nd.op == OP_ADD || nd.op == OP_CONCAT || nd.op == OP_UP2X || nd.op == OP_GAP ||
                      nd.op == OP_MUL || nd.op == OP_DELAY) && nd.act == ACT_NONE;
      s.dy.assign(o.elems(), T(0));
      s.active.assign(o.sites(), 0);
      s.touched.assign(o.sites(), 0);
      if (s.keeps_z) s.z.assign(o.elems(), T(0));
      if (nd.op == OP_MUL) { s.z.assign(o.elems(), T(0)); s.z2.assign(o.elems(), T(0)); }
      if (nd.op == OP_DELAY) s.z.assign(o.elems(), T(0));  // the value emitted so far
      if (nd.op == OP_MAXPOOL) s.pool_in.assign(a.elems(), T(0));
      if (nd.is_output) s.y.assign(o.elems(), T(0));
      if (nd.op == OP_CONV || nd.op == OP_LINEAR) {
        if (nd.w_off < 0 || nd.w_off + (long long)nd.c_out * nd.c_in * nd.k * nd.k > n_w) return 9;
        w_taps[i].resize(size_t(nd.k) * nd.k * nd.c_in * nd.c_out);
        for (int co = 0; co < nd.c_out; ++co)
          for (int ci = 0; ci < nd.c_in; ++ci)
            for (int ky = 0; ky < nd.k; ++ky)
              for (int kx = 0; kx < nd.k; ++kx)
                w_taps[i][((size_t(ky) * nd.k + kx) * nd.c_in + ci) * nd.c_out + co] =
                    T(weights[nd.w_off + ((size_t(co) * nd.c_in + ci) * nd.k + ky) * nd.k + kx]);
      }
      if (nd.op == OP_CONV || nd.op == OP_LINEAR) {
        s.macs_dense_nominal = double(o.sites()) * nd.k * nd.k * nd.c_in * nd.c_out;
        double pairs = 0;
        for (int oy = 0; oy < o.h; ++oy)
          for (int ox = 0; ox < o.w; ++ox)
            for (int ky = 0; ky < nd.k; ++ky)
              for (int kx = 0; kx < nd.k; ++kx) {
                const int iy = oy * nd.stride - nd.pad + ky, ix = ox * nd.stride - nd.pad + kx;
                if (iy >= 0 && iy < a.h && ix >= 0 && ix < a.w) pairs += 1;
              }
        s.macs_dense = pairs * nd.c_in * nd.c_out;
      }
    }
    for (int i = 0; i < n_nodes; ++i)
      if (nodes[i].op == OP_DELAY) {
        const Shape &x = st[nodes[i].in0].shp, &o = st[i].shp;
        if (x.c != o.c || x.h != o.h || x.w != o.w) return 10;
        st[nodes[i].in0].da.assign(o.elems(), T(0));
      }
    x_prev.assign(in.elems(), 0.f);
    dx.assign(in.elems(), T(0));
    s0.assign(in.sites(), 0);
    return 0;
  }

  // ------------------------------------------------------------------ dense pass (definition)
  void dense_forward(const float* x_chw) {
    x_dense.resize(in.elems());
    for (int c = 0; c < in.c; ++c)
      for (size_t p = 0; p < in.sites(); ++p) x_dense[p * in.c + c] = T(x_chw[c * in.sites() + p]);
    for (size_t i = 0; i < nodes.size(); ++i) dense_node(int(i));
  }

  void dense_node(int i) {
    const NodeDesc& nd = nodes[i];
    NodeState<T>& s = st[i];
    const Shape a = shape_of(nd.op == OP_DELAY ? nd.in1 : nd.in0), o = s.shp;
    if (nd.op == OP_DELAY) {
      // X's value at the previous pass: what that pass left in X (a regular pass), or the value
      // emitted so far plus X's last increment (an incremental pass); zero before the first frame
      const NodeState<T>& x = st[nd.in0];
      s.dz.assign(o.elems(), T(0));
      if (!first_pass)
        for (size_t q = 0; q < o.sites(); ++q)
          for (int c = 0; c < o.c; ++c) {
            const size_t e = q * o.c + c;
            s.dz[e] = last_dense ? x.da[e] : s.z[e] + (x.active[q] ? x.dy[e] : T(0));
          }
      s.da = s.dz;
      return;
    }
    const std::vector<T>& xa = dense_of(nd.in0);
    s.dz.assign(o.elems(), T(0));
    switch (nd.op) {
      case OP_CONV:
      case OP_LINEAR: {
#pragma omp parallel for schedule(dynamic, 1)
        for (int oy = 0; oy < o.h; ++oy) {
          std::vector<T> acc(o.c);
          for (int ox = 0; ox < o.w; ++ox) {
            for (int co = 0; co < o.c; ++co) acc[co] = nd.b_off >= 0 ? T(weights[nd.b_off + co]) : T(0);
            for (int ky = 0; ky < nd.k; ++ky) {
              int iy = oy * nd.stride - nd.pad + ky;
              if (iy < 0 || iy >= a.h) continue;  // zero padding
              for (int kx = 0; kx < nd.k; ++kx) {
                int ix = ox * nd.stride - nd.pad + kx;
                if (ix < 0 || ix >= a.w) continue;
                const T* xv = &xa[(size_t(iy) * a.w + ix) * a.c];
                for (int ci = 0; ci < a.c; ++ci) {
                  const T* wr = row(i, nd, ci, ky, kx);
                  T xi = xv[ci];
                  for (int co = 0; co < o.c; ++co) acc[co] += wr[co] * xi;
                }
              }
            }
            std::copy(acc.begin(), acc.end(), &s.dz[(size_t(oy) * o.w + ox) * o.c]);
          }
        }
        break;
      }
      case OP_ADD: {
        const std::vector<T>& xb = dense_of(nd.in1);
        for (size_t e = 0; e < o.elems(); ++e) s.dz[e] = xa[e] + xb[e];
        break;
      }
      case OP_MUL: {
        const std::vector<T>& xb = dense_of(nd.in1);
        for (size_t e = 0; e < o.elems(); ++e) s.dz[e] = xa[e] * xb[e];
        break;
      }
      case OP_ACT: s.dz = xa; break;
      case OP_SPARSIFY: s.dz = xa; break;  // a regular forward pass does not sparsify
      case OP_CONCAT: {
        const Shape b = shape_of(nd.in1);
        const std::vector<T>& xb = dense_of(nd.in1);
        for (size_t p = 0; p < o.sites(); ++p) {
          for (int c = 0; c < a.c; ++c) s.dz[p * o.c + c] = xa[p * a.c + c];
          for (int c = 0; c < b.c; ++c) s.dz[p * o.c + a.c + c] = xb[p * b.c + c];
        }
        break;
      }
      case OP_UP2X:
        for (int oy = 0; oy < o.h; ++oy)
          for (int ox = 0; ox < o.w; ++ox) {
            int y0, y1, x0, x1; double wy0, wy1, wx0, wx1;
            up2_src(oy, a.h, y0, y1, wy0, wy1);
            up2_src(ox, a.w, x0, x1, wx0, wx1);
            for (int c = 0; c < o.c; ++c) {
              auto at = [&](int y, int x) { return xa[(size_t(y) * a.w + x) * a.c + c]; };
              s.dz[(size_t(oy) * o.w + ox) * o.c + c] =
                  T(wy0) * (T(wx0) * at(y0, x0) + T(wx1) * at(y0, x1)) +
                  T(wy1) * (T(wx0) * at(y1, x0) + T(wx1) * at(y1, x1));
            }
          }
        break;
      case OP_MAXPOOL:
        for (int oy = 0; oy < o.h; ++oy)
          for (int ox = 0; ox < o.w; ++ox)
            for (int c = 0; c < o.c; ++c)
              s.dz[(size_t(oy) * o.w + ox) * o.c + c] = window_max(xa, a, nd, oy, ox, c);
        break;
      case OP_GAP:
        for (int c = 0; c < o.c; ++c) {
          T sum = T(0);
          for (size_t p = 0; p < a.sites(); ++p) sum += xa[p * a.c + c];
          s.dz[c] = sum / T(a.sites());
        }
        break;
    }
    s.da.resize(o.elems());
    for (size_t e = 0; e < o.elems(); ++e) s.da[e] = activate<T>(nd.act, s.dz[e]);
  }

  static T window_max(const std::vector<T>& v, const Shape& a, const NodeDesc& nd, int oy, int ox, int c) {
    T m = -std::numeric_limits<T>::infinity();
    for (int ky = 0; ky < nd.k; ++ky) {
      int iy = oy * nd.stride - nd.pad + ky;
      if (iy < 0 || iy >= a.h) continue;
      for (int kx = 0; kx < nd.k; ++kx) {
        int ix = ox * nd.stride - nd.pad + kx;
        if (ix < 0 || ix >= a.w) continue;
        m = std::max(m, v[(size_t(iy) * a.w + ix) * a.c + c]);
      }
    }
    return m;
  }

  // reset: regular forward pass that re-initialises every accumulated tensor, from a zero
  // recurrent state; refresh: the same pass in mid-stream, which keeps the recurrent state
  void reset(const float* x0) { regular_pass(x0, true); }
  void refresh(const float* x) { regular_pass(x, false); }
  void regular_pass(const float* x0, bool first) {
    first_pass = first;
    dense_forward(x0);
    first_pass = false;
    last_dense = true;
    std::copy(x0, x0 + in.elems(), x_prev.begin());
    std::fill(dx.begin(), dx.end(), T(0));
    std::fill(s0.begin(), s0.end(), 0);
    for (size_t i = 0; i < nodes.size(); ++i) {
      NodeState<T>& s = st[i];
      if (s.keeps_z) s.z = s.dz;
      if (nodes[i].op == OP_SPARSIFY) {
        std::fill(s.z.begin(), s.z.end(), T(0));  // residual delta
        if (s.k_fixed >= 0.f) {
          s.k = s.k_fixed;
        } else {
          double sum = 0;
          for (size_t e = 0; e < s.dz.size(); ++e) sum += double(s.dz[e]) * double(s.dz[e]);
          s.k = quantise_step(float(sparsify_tp * std::sqrt(sum / double(s.dz.size()))));
        }
      }
      if (nodes[i].op == OP_MUL) { s.z = dense_of(nodes[i].in0); s.z2 = dense_of(nodes[i].in1); }
      if (nodes[i].op == OP_DELAY) s.z = s.da;
      if (nodes[i].op == OP_MAXPOOL) s.pool_in = dense_of(nodes[i].in0);
      if (nodes[i].is_output) s.y = s.da;
      std::fill(s.dy.begin(), s.dy.end(), T(0));
      std::fill(s.active.begin(), s.active.end(), 0);
      std::fill(s.touched.begin(), s.touched.end(), 0);
      s.macs_site = 0;
    }
    has_state = true;
  }

  // ------------------------------------------------------------------ incremental step
  // Eq.1 on fp32 frames: one binary32 subtraction per element; the frame replaces x_prev.
  void step_frame(const float* xt) {
    for (size_t p = 0; p < in.sites(); ++p) {
      uint8_t any = 0;
      for (int c = 0; c < in.c; ++c) {
        size_t e = c * in.sites() + p;
        float dv = xt[e] - x_prev[e];
        x_prev[e] = xt[e];
        dx[p * in.c + c] = T(dv);
        any |= (dv != 0.0f);
      }
      s0[p] = any;
    }
    propagate();
  }

  // the caller supplies the increment tensor itself
  void step_increment(const float* inc) {
    for (size_t p = 0; p < in.sites(); ++p) {
      uint8_t any = 0;
      for (int c = 0; c < in.c; ++c) {
        size_t e = c * in.sites() + p;
        float dv = inc[e];
        x_prev[e] = x_prev[e] + dv;
        dx[p * in.c + c] = T(dv);
        any |= (dv != 0.0f);
      }
      s0[p] = any;
    }
    propagate();
  }

  void propagate() {
    for (size_t i = 0; i < nodes.size(); ++i) incr_node(int(i));
    last_dense = false;
  }

  // rounding step kept to 8 fraction bits (round to nearest on the 16th mantissa bit)
  static float quantise_step(float k) {
    uint32_t u;
    std::memcpy(&u, &k, 4);
    u = (u + 0x4000u) & 0xffff8000u;
    std::memcpy(&k, &u, 4);
    return k;
  }

  // touched set of a windowed op (conv / max-pool): mark every output that reads an active,
  // in-bounds input site through some tap
  static void touched_windowed(const std::vector<uint8_t>& s_in, const Shape& a, const Shape& o,
                               const NodeDesc& nd, std::vector<uint8_t>& t) {
    std::fill(t.begin(), t.end(), 0);
    for (int iy = 0; iy < a.h; ++iy)
      for (int ix = 0; ix < a.w; ++ix) {
        if (!s_in[size_t(iy) * a.w + ix]) continue;
        for (int ky = 0; ky < nd.k; ++ky) {
          int ny = iy + nd.pad - ky;
          if (ny < 0 || ny % nd.stride) continue;
          int oy = ny / nd.stride;
          if (oy >= o.h) continue;
          for (int kx = 0; kx < nd.k; ++kx) {
            int nx = ix + nd.pad - kx;
            if (nx < 0 || nx % nd.stride) continue;
            int ox = nx / nd.stride;
            if (ox >= o.w) continue;
            t[size_t(oy) * o.w + ox] = 1;
          }
        }
      }
  }

  void incr_node(int i) {
    const NodeDesc& nd = nodes[i];
    NodeState<T>& s = st[i];
    if (nd.op == OP_DELAY) {
      // X has not been visited in this pass yet: its increment and mask are those of the
      // previous step; after a regular pass the increment is X's value minus what was emitted
      const NodeState<T>& x = st[nd.in0];
      const Shape o = s.shp;
      for (size_t q = 0; q < o.sites(); ++q) {
        const uint8_t on = last_dense ? 1 : x.active[q];
        for (int c = 0; c < o.c; ++c) {
          const size_t e = q * o.c + c;
          const T inc = !on ? T(0) : (last_dense ? x.da[e] - s.z[e] : x.dy[e]);
          s.dy[e] = inc;
          s.z[e] += inc;
          if (nd.is_output) s.y[e] += inc;
        }
        s.active[q] = s.touched[q] = on;
      }
      s.macs_site = 0;
      return;
    }
    const Shape a = shape_of(nd.in0), o = s.shp;
    const std::vector<T>& da = dy_of(nd.in0);
    const std::vector<uint8_t>& sa = set_of(nd.in0);
    // clear last step's increment on its old support
    for (size_t q = 0; q < o.sites(); ++q)
      if (s.touched[q]) std::fill(&s.dy[q * o.c], &s.dy[q * o.c] + o.c, T(0));
    if (nd.op == OP_SPARSIFY) {  // Eq.3-8 under the reading in the header
      const T k = T(s.k);
      for (size_t q = 0; q < o.sites(); ++q) {
        s.touched[q] = sa[q];
        s.active[q] = 0;
        if (!sa[q]) continue;
        uint8_t nz = 0;
        for (int c = 0; c < o.c; ++c) {
          const size_t e = q * o.c + c;
          T y = da[e];
          // An element whose input increment is zero emits nothing and keeps its residual: with
          // -k/2 <= delta < k/2 (the bound the section asks of the residual) Eq.6-7 give
          // floor(0.5 + delta / k) = 0 for it, and taking that for granted keeps the layer
          // independent of the mask (which may cover such an element or not).  The zero test is the
          // binary32 one of the masks.
          if (k > T(0) && float(da[e]) != 0.0f) {
            const T x_corr = s.z[e] + da[e];
            y = k * std::floor(T(0.5) + x_corr / k);
            s.z[e] = x_corr - y;
          }
          s.dy[e] = y;
          nz |= (float(y) != 0.0f);
        }
        s.active[q] = nz;
        if (!nz) std::fill(&s.dy[q * o.c], &s.dy[q * o.c] + o.c, T(0));
        if (nz && nd.is_output)  // Eq.2
          for (int c = 0; c < o.c; ++c) s.y[q * o.c + c] += s.dy[q * o.c + c];
      }
      s.macs_site = 0;
      return;
    }
    std::vector<T> v;  // linear-part increment at touched sites, HWC dense-addressed
    v.assign(o.elems(), T(0));
    std::vector<float> v32;  // max-pool only: the increment formed from binary32-rounded maxima
    s.macs_site = 0;

    switch (nd.op) {
      case OP_CONV:
      case OP_LINEAR: {
        touched_windowed(sa, a, o, nd, s.touched);
        std::vector<int> tl;
        for (size_t q = 0; q < o.sites(); ++q) if (s.touched[q]) tl.push_back(int(q));
        double macs = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : macs)
        for (size_t n = 0; n < tl.size(); ++n) {
          int q = tl[n], oy = q / o.w, ox = q % o.w;
          T* acc = &v[size_t(q) * o.c];
          for (int ky = 0; ky < nd.k; ++ky) {
            int iy = oy * nd.stride - nd.pad + ky;
            if (iy < 0 || iy >= a.h) continue;
            for (int kx = 0; kx < nd.k; ++kx) {
              int ix = ox * nd.stride - nd.pad + kx;
              if (ix < 0 || ix >= a.w) continue;
              size_t p = size_t(iy) * a.w + ix;
              if (!sa[p]) continue;  // all-zero site: contributes nothing
              macs += double(a.c) * o.c;
              const T* xv = &da[p * a.c];
              for (int ci = 0; ci < a.c; ++ci) {
                const T* wr = row(i, nd, ci, ky, kx);
                T xi = xv[ci];
                for (int co = 0; co < o.c; ++co) acc[co] += wr[co] * xi;
              }
            }
          }
        }
        s.macs_site = macs;
        break;
      }
      case OP_ADD: {  // Eq.11
        const std::vector<T>& db = dy_of(nd.in1);
        const std::vector<uint8_t>& sb = set_of(nd.in1);
        for (size_t q = 0; q < o.sites(); ++q) {
          s.touched[q] = sa[q] | sb[q];
          if (!s.touched[q]) continue;
          for (int c = 0; c < o.c; ++c) v[q * o.c + c] = da[q * o.c + c] + db[q * o.c + c];
        }
        break;
      }
      case OP_MUL: {  // Eq.15-17
        const std::vector<T>& db = dy_of(nd.in1);
        const std::vector<uint8_t>& sb = set_of(nd.in1);
        for (size_t q = 0; q < o.sites(); ++q) {
          s.touched[q] = sa[q] | sb[q];  // Eq.16
          if (!s.touched[q]) continue;
          for (int c = 0; c < o.c; ++c) {
            const size_t e = q * o.c + c;
            const T x1 = sa[q] ? da[e] : T(0), x2 = sb[q] ? db[e] : T(0);
            v[e] = (s.z[e] + x1) * x2 + s.z2[e] * x1;  // Eq.15, accumulators of the previous step
            s.z[e] += x1;                              // Eq.17
            s.z2[e] += x2;
          }
        }
        break;
      }
      case OP_ACT:
        for (size_t q = 0; q < o.sites(); ++q) {
          s.touched[q] = sa[q];
          if (!s.touched[q]) continue;
          for (int c = 0; c < o.c; ++c) v[q * o.c + c] = da[q * o.c + c];
        }
        break;
      case OP_CONCAT: {
        const Shape b = shape_of(nd.in1);
        const std::vector<T>& db = dy_of(nd.in1);
        const std::vector<uint8_t>& sb = set_of(nd.in1);
        for (size_t q = 0; q < o.sites(); ++q) {
          s.touched[q] = sa[q] | sb[q];
          if (!s.touched[q]) continue;
          for (int c = 0; c < a.c; ++c) v[q * o.c + c] = da[q * a.c + c];
          for (int c = 0; c < b.c; ++c) v[q * o.c + a.c + c] = db[q * b.c + c];
        }
        break;
      }
      case OP_UP2X:  // linear => Eq.10 on the increment
        for (int oy = 0; oy < o.h; ++oy)
          for (int ox = 0; ox < o.w; ++ox) {
            int y0, y1, x0, x1; double wy0, wy1, wx0, wx1;
            up2_src(oy, a.h, y0, y1, wy0, wy1);
            up2_src(ox, a.w, x0, x1, wx0, wx1);
            size_t q = size_t(oy) * o.w + ox;
            s.touched[q] = sa[size_t(y0) * a.w + x0] | sa[size_t(y0) * a.w + x1] |
                           sa[size_t(y1) * a.w + x0] | sa[size_t(y1) * a.w + x1];
            if (!s.touched[q]) continue;
            for (int c = 0; c < o.c; ++c) {
              auto at = [&](int y, int x) { return da[(size_t(y) * a.w + x) * a.c + c]; };
              v[q * o.c + c] = T(wy0) * (T(wx0) * at(y0, x0) + T(wx1) * at(y0, x1)) +
                               T(wy1) * (T(wx0) * at(y1, x0) + T(wx1) * at(y1, x1));
            }
          }
        break;
      case OP_MAXPOOL: {
        // windowed nonlinearity with accumulated input (Eq.12 generalised): the output
        // increment is max over the updated window minus max over the old window
        touched_windowed(sa, a, o, nd, s.touched);
        std::vector<T> old_max(o.elems(), T(0));
        v32.assign(o.elems(), 0.f);
        for (int oy = 0; oy < o.h; ++oy)
          for (int ox = 0; ox < o.w; ++ox) {
            size_t q = size_t(oy) * o.w + ox;
            if (!s.touched[q]) continue;
            for (int c = 0; c < o.c; ++c) old_max[q * o.c + c] = window_max(s.pool_in, a, nd, oy, ox, c);
          }
        for (size_t p = 0; p < a.sites(); ++p)
          if (sa[p])
            for (int c = 0; c < a.c; ++c) s.pool_in[p * a.c + c] += da[p * a.c + c];
        for (int oy = 0; oy < o.h; ++oy)
          for (int ox = 0; ox < o.w; ++ox) {
            size_t q = size_t(oy) * o.w + ox;
            if (!s.touched[q]) continue;
            for (int c = 0; c < o.c; ++c) {
              T new_max = window_max(s.pool_in, a, nd, oy, ox, c);
              v[q * o.c + c] = new_max - old_max[q * o.c + c];
              v32[q * o.c + c] = float(new_max) - float(old_max[q * o.c + c]);
            }
          }
        break;
      }
      case OP_GAP: {
        bool any = false;
        for (size_t p = 0; p < a.sites(); ++p) any |= bool(sa[p]);
        s.touched[0] = any;
        if (any)
          for (int c = 0; c < o.c; ++c) {
            T sum = T(0);
            for (size_t p = 0; p < a.sites(); ++p)
              if (sa[p]) sum += da[p * a.c + c];
            v[c] = sum / T(a.sites());
          }
        break;
      }
    }

    // accumulate, apply the activation increment (Eq.12-14) and derive the active set
    for (size_t q = 0; q < o.sites(); ++q) {
      s.active[q] = 0;
      if (!s.touched[q]) continue;
      uint8_t nz = 0;
      for (int c = 0; c < o.c; ++c) {
        size_t e = q * o.c + c;
        T out = v[e];
        // out32: the same increment evaluated on binary32-rounded operands.  Whether a site is
        // kept is an integer decided by floating point; it is taken in binary32, the precision
        // the cached tensors of the method are held in.
        float out32 = v32.empty() ? float(v[e]) : v32[e];
        if (s.keeps_z) {
          T z_old = s.z[e];
          T z_new = z_old + v[e];
          s.z[e] = z_new;
          if (nd.act != ACT_NONE) {
            out = activate<T>(nd.act, z_new) - activate<T>(nd.act, z_old);
            out32 = activate<float>(nd.act, float(z_new)) - activate<float>(nd.act, float(z_old));
          }
        }
        s.dy[e] = out;
        nz |= (out32 != 0.0f);
      }
      s.active[q] = s.structural ? 1 : nz;
      if (!s.active[q]) std::fill(&s.dy[q * o.c], &s.dy[q * o.c] + o.c, T(0));
    }
    if (nd.is_output)  // Eq.2
      for (size_t q = 0; q < o.sites(); ++q)
        if (s.active[q])
          for (int c = 0; c < o.c; ++c) s.y[q * o.c + c] += s.dy[q * o.c + c];
  }
};

struct Handle {
  int fp32;
  Net<double> d;
  Net<float> f;
};

template <class T>
void copy_out(const std::vector<T>& v, double* dst) {
  for (size_t i = 0; i < v.size(); ++i) dst[i] = double(v[i]);
}

template <class T>
long long get_tensor(Net<T>& n, int node, int kind, double* dst) {
  // kind: 0 z, 1 dy, 2 y (outputs), 3 dense pre-activation, 4 dense value, 5 pool_in, 6 z2
  if (node < 0) {
    if (kind != 1) return -1;
    if (dst) copy_out(n.dx, dst);
    return (long long)n.dx.size();
  }
  NodeState<T>& s = n.st[node];
  const std::vector<T>* v = nullptr;
  switch (kind) {
    case 0: v = &s.z; break;
    case 1: v = &s.dy; break;
    case 2: v = &s.y; break;
    case 3: v = &s.dz; break;
    case 4: v = &s.da; break;
    case 5: v = &s.pool_in; break;
    case 6: v = &s.z2; break;
    default: return -1;
  }
  if (dst) copy_out(*v, dst);
  return (long long)v->size();
}

template <class T>
long long get_set(Net<T>& n, int node, int kind, uint8_t* dst) {
  // kind: 0 active set S, 1 touched set T   (dense H*W byte mask)
  const std::vector<uint8_t>& v = node < 0 ? n.s0 : (kind == 0 ? n.st[node].active : n.st[node].touched);
  if (dst) std::copy(v.begin(), v.end(), dst);
  return (long long)v.size();
}

}  // namespace

extern "C" {

// desc: n_nodes x 12 int32 {op, act, in0, in1, c_in, c_out, k, stride, pad, w_off, b_off, is_output}
void* evo_create(int n_nodes, const int* desc, const double* weights, long long n_weights,
                 int in_c, int in_h, int in_w, int fp32_state, double sparsify_tp) {
  Handle* h = new Handle();
  h->fp32 = fp32_state;
  h->d.sparsify_tp = sparsify_tp;
  h->f.sparsify_tp = sparsify_tp;
  int rc = fp32_state ? h->f.init(n_nodes, desc, weights, n_weights, in_c, in_h, in_w)
                      : h->d.init(n_nodes, desc, weights, n_weights, in_c, in_h, in_w);
  if (rc) { delete h; return nullptr; }
  return h;
}
void evo_destroy(void* h) { delete (Handle*)h; }
void evo_dense_forward(void* h, const float* x) {
  Handle* p = (Handle*)h;
  if (p->fp32) p->f.dense_forward(x); else p->d.dense_forward(x);
}
void evo_reset(void* h, const float* x0) {
  Handle* p = (Handle*)h;
  if (p->fp32) p->f.reset(x0); else p->d.reset(x0);
}
void evo_refresh(void* h, const float* x) {
  Handle* p = (Handle*)h;
  if (p->fp32) p->f.refresh(x); else p->d.refresh(x);
}
void evo_step_frame(void* h, const float* xt) {
  Handle* p = (Handle*)h;
  if (p->fp32) p->f.step_frame(xt); else p->d.step_frame(xt);
}
void evo_step_increment(void* h, const float* inc) {
  Handle* p = (Handle*)h;
  if (p->fp32) p->f.step_increment(inc); else p->d.step_increment(inc);
}
long long evo_get_tensor(void* h, int node, int kind, double* dst) {
  Handle* p = (Handle*)h;
  return p->fp32 ? get_tensor(p->f, node, kind, dst) : get_tensor(p->d, node, kind, dst);
}
long long evo_get_set(void* h, int node, int kind, uint8_t* dst) {
  Handle* p = (Handle*)h;
  return p->fp32 ? get_set(p->f, node, kind, dst) : get_set(p->d, node, kind, dst);
}
void evo_get_shape(void* h, int node, int* chw) {
  Handle* p = (Handle*)h;
  Shape s = p->fp32 ? p->f.shape_of(node) : p->d.shape_of(node);
  chw[0] = s.c; chw[1] = s.h; chw[2] = s.w;
}
void evo_get_x_prev(void* h, float* dst) {
  Handle* p = (Handle*)h;
  const std::vector<float>& v = p->fp32 ? p->f.x_prev : p->d.x_prev;
  std::copy(v.begin(), v.end(), dst);
}
// rounding step of a sparsification node (0 for other nodes)
float evo_get_step(void* h, int node) {
  Handle* p = (Handle*)h;
  return p->fp32 ? p->f.st[node].k : p->d.st[node].k;
}
// Multiply-accumulate counts of a conv / linear node (zeros for other nodes), out[4]:
//   [0] executed by the last step at site granularity (macs_site)
//   [1] executed by the last step when whole mask tiles of th x tw outputs are computed: the
//       number of tiles holding at least one touched output * th * tw * k * k * c_in * c_out
//       ("Convolution on Sparse Inputs": filter applications are skipped per all-zero section)
//   [2] a regular forward pass, padding taps not counted (macs_dense)
//   [3] a regular forward pass, outputs * k * k * c_in * c_out (macs_dense_nominal)
void evo_get_macs(void* h, int node, int th, int tw, double* out) {
  Handle* p = (Handle*)h;
  auto fill = [&](auto& net) {
    auto& s = net.st[node];
    const NodeDesc& nd = net.nodes[node];
    out[0] = s.macs_site; out[2] = s.macs_dense; out[3] = s.macs_dense_nominal; out[1] = 0;
    if (nd.op != OP_CONV && nd.op != OP_LINEAR) return;
    const int ty = (s.shp.h + th - 1) / th, tx = (s.shp.w + tw - 1) / tw;
    std::vector<uint8_t> hit(size_t(ty) * tx, 0);
    for (int y = 0; y < s.shp.h; ++y)
      for (int x = 0; x < s.shp.w; ++x)
        if (s.touched[size_t(y) * s.shp.w + x]) hit[size_t(y / th) * tx + x / tw] = 1;
    double tiles = 0;
    for (uint8_t v : hit) tiles += v;
    out[1] = tiles * th * tw * nd.k * nd.k * nd.c_in * nd.c_out;
  };
  if (p->fp32) fill(p->f); else fill(p->d);
}

}  // extern "C"
