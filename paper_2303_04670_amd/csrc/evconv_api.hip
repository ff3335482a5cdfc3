// Host side of the C ABI declared in include/evconv.h: description checking, workspace
// layout, weight re-layout, and the per-step launch sequence.  No computation of the method
// happens on the host; every step of the path is a kernel launch on the caller's stream.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/evconv.h"
#include "evconv_kernels.h"

using namespace evk;

namespace {

thread_local std::string g_create_error;

// Workspace of evconv_create_static: one array per GPU, part of the loaded code object, so a net
// built in it needs no device allocation by anybody.  In host code the array's name is only a
// handle for hipGetSymbolAddress; the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[EVCONV_STATIC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_scratch_ptr[kMaxDevices] = {};       // device address of `scratch` on each device
evconv_net* g_static_owner[kMaxDevices] = {};  // the live net that occupies it, if any

enum KernelKind { kKernConvValu = 0, kKernConvMfmaF32, kKernElementwise, kKernGap, kKernPool, kKernConvMfmaBf16,
                  kKernConvNarrow, kKernConvMfmaSplit, kKernConvPointwise, kKernDelay };
const char* const kKernelNames[] = {"conv_valu_f32", "conv_mfma_f32", "elementwise", "global_avgpool",
                                    "maxpool", "conv_mfma_bf16", "conv_narrow_mfma_f32", "conv_mfma_f32_split_bf16x3", "conv_pointwise_f32",
                                    "delay"};

// fp32 -> bf16 bits, round to nearest even
uint16_t to_bf16(float x) {
  uint32_t u;
  memcpy(&u, &x, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

struct NodePlan {
  evconv_node_desc d;
  Geo ga, gb, go;
  bool keeps_z = false, structural = false;
  int kernel = 0;
  int c_out_pad = 0;
  int fused_into = -1;      // ADD or SPARSIFY node executed in the epilogue of that conv node
  int fused_sp = -1;        // conv node: the SPARSIFY node it executes behind its last epilogue stage
  int n_fused = 0;          // conv node: ADD nodes it executes, in order
  int fused_nodes[kMaxFusedAdds] = {-1, -1};
  int gather_fused_into = -1;  // UPSAMPLE node computed inside the gather of that conv node, never stored
  int upsampled_from = -2;     // conv node: the node (-1: network input) whose x2 up-sampling it reads through
                               // its gather, its in0 being the folded UPSAMPLE node; -2: none
  // conv node reading through an up-sampling: the up-sampling folded into per-phase weights
  // away from the image border (ConvParams::fold_list); room is reserved whenever in0 is an
  // up-sampling and the taps are 5 x 5, used if the planner folds that up-sampling into this conv
  size_t off_w_fold = 0, off_fold_list = 0;
  void* w_fold = nullptr;
  int* fold_list = nullptr;
  int fold_k = 0, fold_base[2] = {0, 0};
  // workspace offsets (bytes); resolved to pointers at create
  size_t off_step = 0;      // SPARSIFY: device scalar k
  size_t off_z2 = 0;        // MUL: accumulated second factor
  float* z2 = nullptr;
  size_t off_occ_saved = 0;  // DELAY: S_out words of the delayed node as the previous step left them
  uint64_t* occ_saved = nullptr;
  float* step = nullptr;
  float step_fixed = -1.0f; // >= 0: k supplied by the description
  size_t off_z = 0, off_out = 0, off_pool = 0, off_occ = 0, off_touched = 0, off_idx = 0, off_count = 0,
         off_bitmap = 0, off_w = 0, off_bias = 0, off_y = 0, off_dy = 0;
  float *z = nullptr, *out = nullptr, *pool_in = nullptr, *bias = nullptr, *y = nullptr, *dy = nullptr;
  void* w = nullptr;
  uint64_t *occ = nullptr, *touched = nullptr, *bitmap = nullptr;
  int32_t *idx = nullptr, *count = nullptr;
};

struct Layout {
  std::vector<NodePlan> nodes;
  Geo gin;
  size_t off_x_prev = 0, off_dx = 0, off_occ_in = 0, off_idx_in = 0, off_count_in = 0, off_bitmap_in = 0;
  size_t off_occ_nodes = 0, n_occ_words = 0;  // contiguous occupancy region of all nodes
  size_t off_sets = 0, off_rms = 0;
  size_t stride = 0;   // bytes of one stream's state (the weights live in stream 0's copy)
  int n_streams = 1;
  size_t total = 0;
  int max_ty = 0;
};

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Bump {
  size_t cur = 0;
  size_t take(size_t bytes) {
    size_t o = cur;
    cur = align_up(cur + bytes);
    return o;
  }
};

evconv_status fail(std::string* err, evconv_status st, const std::string& msg) {
  if (err) *err = msg;
  return st;
}

// Checks the description and lays the workspace out.  Pure host arithmetic.
evconv_status make_layout(const evconv_net_desc* desc, size_t weight_bytes, bool check_weights, Layout* L,
                          std::string* err) {
  if (!desc || !desc->nodes) return fail(err, EVCONV_ERR_INVALID_ARG, "null description");
  if (desc->abi_version != EVCONV_ABI_VERSION) return fail(err, EVCONV_ERR_BAD_DESC, "abi_version mismatch");
  if (desc->n_nodes <= 0) return fail(err, EVCONV_ERR_BAD_DESC, "n_nodes must be positive");
  if (desc->in_c <= 0 || desc->in_h <= 0 || desc->in_w <= 0) return fail(err, EVCONV_ERR_SHAPE, "bad input shape");
  if (desc->flags & ~(EVCONV_FLAG_NO_FUSION | EVCONV_FLAG_NO_FOLD | EVCONV_FLAG_FORCE_VALU))
    return fail(err, EVCONV_ERR_INVALID_ARG, "unknown bits in flags");
  if (!(desc->sparsify_tp >= 0.0f)) return fail(err, EVCONV_ERR_INVALID_ARG, "sparsify_tp must be >= 0");
  if (desc->n_streams < 0 || desc->n_streams > 256) return fail(err, EVCONV_ERR_INVALID_ARG, "n_streams must be in [0, 256]");
  if ((long long)desc->in_h * desc->in_w > (1ll << 30)) return fail(err, EVCONV_ERR_SHAPE, "input too large");

  L->gin = make_geo(desc->in_c, desc->in_h, desc->in_w);
  L->nodes.resize(desc->n_nodes);
  L->max_ty = L->gin.ty;
  Bump b;
  // occupancy words of all nodes first, contiguous: cleared in one sweep at the start of a step
  L->off_occ_nodes = b.cur;
  std::vector<size_t> occ_word_off(desc->n_nodes);
  size_t words = 0;
  for (int i = 0; i < desc->n_nodes; ++i) {
    const evconv_node_desc& d = desc->nodes[i];
    NodePlan& n = L->nodes[i];
    n.d = d;
    char where[64];
    snprintf(where, sizeof where, "node %d: ", i);
    if (d.op < 0 || d.op > EVCONV_OP_DELAY) return fail(err, EVCONV_ERR_INVALID_ARG, std::string(where) + "bad op");
    if (d.act < 0 || d.act > EVCONV_ACT_ONE_MINUS) return fail(err, EVCONV_ERR_INVALID_ARG, std::string(where) + "bad act");
    const bool delay = d.op == EVCONV_OP_DELAY;
    if (delay) {
      // in0: the later node whose previous-step value this is; in1: an earlier node of its size
      if (d.in0 <= i || d.in0 >= desc->n_nodes) return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "DELAY: in0 must be a later node");
      if (d.in1 < -1 || d.in1 >= i) return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "DELAY: in1 is not an earlier node");
      if (d.act != EVCONV_ACT_NONE) return fail(err, EVCONV_ERR_UNSUPPORTED, std::string(where) + "DELAY takes no activation");
      if (d.c_out <= 0) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "c_out must be positive");
    } else if (d.in0 < -1 || d.in0 >= i) {
      return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "in0 is not an earlier node");
    }
    const bool two = d.op == EVCONV_OP_ADD || d.op == EVCONV_OP_CONCAT || d.op == EVCONV_OP_MUL;
    if (two && (d.in1 < -1 || d.in1 >= i)) return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "in1 is not an earlier node");
    if (delay) {
      n.ga = d.in1 < 0 ? L->gin : L->nodes[d.in1].go;
      n.ga = make_geo(d.c_out, n.ga.h, n.ga.w);
    } else {
      n.ga = d.in0 < 0 ? L->gin : L->nodes[d.in0].go;
    }
    n.gb = two ? (d.in1 < 0 ? L->gin : L->nodes[d.in1].go) : n.ga;
    int c = n.ga.c, h = n.ga.h, w = n.ga.w;
    switch (d.op) {
      case EVCONV_OP_CONV2D:
      case EVCONV_OP_LINEAR:
      case EVCONV_OP_MAXPOOL: {
        int k = d.kh, s = d.stride, pad = d.pad;
        if (d.op == EVCONV_OP_LINEAR) {
          if (h != 1 || w != 1) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "LINEAR needs a 1 x 1 input");
          k = 1; s = 1; pad = 0;
          n.d.kh = n.d.kw = 1; n.d.stride = 1; n.d.pad = 0;
        } else {
          if (d.kh != d.kw || k < 1 || k > 7) return fail(err, EVCONV_ERR_UNSUPPORTED, std::string(where) + "kernel must be square, 1..7");
          if (s < 1 || s > 2) return fail(err, EVCONV_ERR_UNSUPPORTED, std::string(where) + "stride must be 1 or 2");
          if (pad < 0 || pad >= k) return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "pad must be in [0, k)");
        }
        if (d.op == EVCONV_OP_MAXPOOL) {
          if (d.act != EVCONV_ACT_NONE) return fail(err, EVCONV_ERR_UNSUPPORTED, std::string(where) + "MAXPOOL takes no activation");
        } else {
          if (d.c_in != c) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "c_in does not match the input node");
          if (d.c_out <= 0) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "c_out must be positive");
          if (d.wdtype != EVCONV_F32 && d.wdtype != EVCONV_BF16 && d.wdtype != EVCONV_F32_SPLIT) return fail(err, EVCONV_ERR_INVALID_ARG, std::string(where) + "bad wdtype");
          const size_t wb = (size_t)d.c_out * d.c_in * k * k * sizeof(float);
          if (d.weight_off < 0 || (d.weight_off & 3)) return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "bad weight_off");
          if (check_weights && (size_t)d.weight_off + wb > weight_bytes) return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "weights out of range");
          if (d.bias_off >= 0 && ((d.bias_off & 3) || (check_weights && (size_t)d.bias_off + d.c_out * sizeof(float) > weight_bytes)))
            return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "bias out of range");
          c = d.c_out;
        }
        const int ho = (h + 2 * pad - k) / s + 1, wo = (w + 2 * pad - k) / s + 1;
        if (h + 2 * pad < k || w + 2 * pad < k || ho <= 0 || wo <= 0) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "empty output");
        h = ho; w = wo;
        break;
      }
      case EVCONV_OP_ADD:
        if (n.gb.c != c || n.gb.h != h || n.gb.w != w) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "ADD inputs differ in shape");
        break;
      case EVCONV_OP_MUL:
        if (n.gb.c != c || n.gb.h != h || n.gb.w != w) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "MUL inputs differ in shape");
        if (d.act != EVCONV_ACT_NONE) return fail(err, EVCONV_ERR_UNSUPPORTED, std::string(where) + "MUL takes no activation");
        break;
      case EVCONV_OP_CONCAT:
        if (n.gb.h != h || n.gb.w != w) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "CONCAT inputs differ in size");
        c += n.gb.c;
        break;
      case EVCONV_OP_UPSAMPLE_BILINEAR2X: h *= 2; w *= 2; break;
      case EVCONV_OP_GLOBAL_AVGPOOL: h = 1; w = 1; break;
      case EVCONV_OP_ACT: break;
      case EVCONV_OP_DELAY: break;  // shape of in1 with c_out channels; checked against in0 below
      case EVCONV_OP_SPARSIFY:
        if (d.act != EVCONV_ACT_NONE) return fail(err, EVCONV_ERR_UNSUPPORTED, std::string(where) + "SPARSIFY takes no activation");
        if (d.weight_off >= 0 && ((d.weight_off & 3) || (check_weights && (size_t)d.weight_off + 4 > weight_bytes)))
          return fail(err, EVCONV_ERR_BAD_DESC, std::string(where) + "step value out of range");
        break;
    }
    if ((long long)h * w > (1ll << 30)) return fail(err, EVCONV_ERR_SHAPE, std::string(where) + "output too large");
    n.go = make_geo(c, h, w);
    if (n.go.ty > L->max_ty) L->max_ty = n.go.ty;
    const bool lin = d.op == EVCONV_OP_CONV2D || d.op == EVCONV_OP_LINEAR;
    n.keeps_z = (lin || d.op == EVCONV_OP_GLOBAL_AVGPOOL || d.op == EVCONV_OP_ACT ||
                 d.op == EVCONV_OP_SPARSIFY || d.op == EVCONV_OP_MUL || d.op == EVCONV_OP_DELAY ||
                 d.act != EVCONV_ACT_NONE) &&
                d.op != EVCONV_OP_MAXPOOL;
    n.structural = (d.op == EVCONV_OP_ADD || d.op == EVCONV_OP_CONCAT || d.op == EVCONV_OP_UPSAMPLE_BILINEAR2X ||
                    d.op == EVCONV_OP_GLOBAL_AVGPOOL || d.op == EVCONV_OP_MUL || d.op == EVCONV_OP_DELAY) &&
                   d.act == EVCONV_ACT_NONE;
    if (lin) {
      n.kernel = kKernConvValu;
      n.c_out_pad = (d.c_out + 31) / 32 * 32;
    } else if (d.op == EVCONV_OP_GLOBAL_AVGPOOL) n.kernel = kKernGap;
    else if (d.op == EVCONV_OP_MAXPOOL) n.kernel = kKernPool;
    else if (d.op == EVCONV_OP_DELAY) n.kernel = kKernDelay;
    else n.kernel = kKernElementwise;
    occ_word_off[i] = words;
    words += 2 * (size_t)n.go.tiles();
  }
  for (int i = 0; i < desc->n_nodes; ++i) {
    const NodePlan& n = L->nodes[i];
    if (n.d.op != EVCONV_OP_DELAY) continue;
    const Geo& x = L->nodes[n.d.in0].go;
    if (x.c != n.go.c || x.h != n.go.h || x.w != n.go.w) {
      char where[96];
      snprintf(where, sizeof where, "node %d: DELAY shape differs from that of node %d", i, n.d.in0);
      return fail(err, EVCONV_ERR_SHAPE, where);
    }
  }
  L->n_occ_words = words;
  b.take(words * sizeof(uint64_t));
  for (int i = 0; i < desc->n_nodes; ++i) {
    NodePlan& n = L->nodes[i];
    n.off_occ = L->off_occ_nodes + occ_word_off[i] * sizeof(uint64_t);
    n.off_touched = n.off_occ + (size_t)n.go.tiles() * sizeof(uint64_t);
  }
  // input stage
  const size_t in_elems = (size_t)L->gin.c * L->gin.sites();
  L->off_x_prev = b.take(in_elems * 4);
  L->off_dx = b.take(in_elems * 4);
  L->off_occ_in = b.take((size_t)L->gin.tiles() * 8);
  L->off_idx_in = b.take((size_t)L->gin.sites() * 4);
  L->off_count_in = b.take(4);
  L->off_bitmap_in = b.take(((size_t)L->gin.tiles() + 63) / 64 * 8);
  for (int i = 0; i < desc->n_nodes; ++i) {
    NodePlan& n = L->nodes[i];
    const size_t elems = (size_t)n.go.c * n.go.sites();
    if (n.keeps_z || n.d.op == EVCONV_OP_MAXPOOL) n.off_z = b.take(elems * 4);
    if (n.d.op == EVCONV_OP_SPARSIFY) n.off_step = b.take(4);
    if (n.d.op == EVCONV_OP_MUL) n.off_z2 = b.take(elems * 4);
    if (n.d.op == EVCONV_OP_DELAY) n.off_occ_saved = b.take((size_t)n.go.tiles() * 8);
    if (n.d.op == EVCONV_OP_MAXPOOL) n.off_pool = b.take((size_t)n.ga.c * n.ga.sites() * 4);
    n.off_out = b.take(elems * 4);
    n.off_idx = b.take((size_t)n.go.sites() * 4);
    n.off_count = b.take(4);
    n.off_bitmap = b.take(((size_t)n.go.tiles() + 63) / 64 * 8);
    if (n.d.op == EVCONV_OP_CONV2D || n.d.op == EVCONV_OP_LINEAR) {
      const int k = n.d.kh;
      // room for input channels padded to whole chunks (at most 64) or a padded flattened contraction
      n.off_w = b.take(std::max(((size_t)k * k * ((n.d.c_in + 63) / 64 * 64) + 16) * n.c_out_pad * 4,
                                conv_narrow_weight_floats(n.c_out_pad) * 4));  // (the narrow-input kernel's per-lane layout)
      if (n.d.bias_off >= 0) n.off_bias = b.take((size_t)n.d.c_out * 4);
      if (n.d.op == EVCONV_OP_CONV2D && k == 5 && n.d.stride == 1 && n.d.pad == 2 && n.d.in0 >= 0 &&
          L->nodes[n.d.in0].d.op == EVCONV_OP_UPSAMPLE_BILINEAR2X) {
        // four phases x (4 x 4 taps) x input channels padded to 32 (see the planner in evconv_create)
        n.off_w_fold = b.take((size_t)4 * 16 * ((n.d.c_in + 31) / 32 * 32) * n.c_out_pad * 4);
        n.off_fold_list = b.take((size_t)n.go.tiles() * 4);
      }
    }
    if (n.d.is_output) {
      n.off_y = b.take(elems * 4);
      n.off_dy = b.take(elems * 4);
    }
  }
  L->off_rms = b.take(sizeof(float) * kRmsBlocks);
  L->off_sets = b.take(sizeof(SetDesc) * (size_t)(desc->n_nodes + 1));
  L->stride = (b.cur + 255) / 256 * 256;  // one stream's copy of everything
  L->n_streams = desc->n_streams > 0 ? desc->n_streams : 1;
  L->total = L->stride * (size_t)L->n_streams;
  return EVCONV_OK;
}

}  // namespace

struct evconv_net {
  Layout L;
  float sparsify_tp = 0.0f;
  float* rms_partial = nullptr;
  std::vector<evconv_node_desc> desc_nodes;
  char* ws = nullptr;
  hipStream_t stream = nullptr;
  int mode = EVCONV_MODE_INCREMENTAL;
  uint32_t flags = 0;
  bool has_sparsify = false;  // some SPARSIFY node has a nonzero rounding step
  // AUTO mode: windows of kAutoProbe steps are timed in each mode with an event pair; the faster
  // mode then runs for kAutoHold steps
  int auto_choice = EVCONV_MODE_INCREMENTAL;
  int auto_phase = 0;         // 0: timing incremental, 1: timing dense recompute, 2: holding auto_choice
  int auto_count = 0;         // steps done in the current phase
  bool auto_pending = false;  // both windows are recorded, their events may not have completed yet
  hipEvent_t auto_ev[4] = {nullptr, nullptr, nullptr, nullptr};
  int refresh_period = 0, since_refresh = 0;
  bool has_state = false;
  int static_device = -1;   // >= 0: the net lives in that device's static workspace
  bool last_dense = true;   // the previous pass was a regular forward pass (DELAY nodes)
  bool zero_state = false;  // the pass being enqueued starts from the zero recurrent state (reset)
  Streams st{0, 1};
  size_t in_stride = 0;
  std::string err;
  std::vector<int> outputs;
  float *x_prev = nullptr, *dx = nullptr;
  uint64_t *occ_in = nullptr, *bitmap_in = nullptr, *occ_nodes = nullptr;
  int32_t *idx_in = nullptr, *count_in = nullptr;
  SetDesc* sets_dev = nullptr;
  // optional per-node timing with HIP events on the net's stream
  bool prof = false;
  std::vector<hipEvent_t> prof_ev;
  std::vector<int> prof_node;
  std::vector<double> node_ms;
  std::vector<long long> node_launches;
};

namespace {

evconv_status hip_fail(evconv_net* net, hipError_t e, const char* what) {
  net->err = std::string(what) + ": " + hipGetErrorString(e);
  return EVCONV_ERR_HIP;
}

// kPassRefresh: the refresh step of "Drift Errors" in mid-stream: a reset that keeps the recurrent
// state and returns dy = y(n) - y(n-1), so that Eq.2 holds across it
enum PassKind { kPassStep = 0, kPassReset = 1, kPassRecompute = 2, kPassRefresh = 3 };
constexpr int kAutoProbe = 4, kAutoHold = 256;

// Enqueues one pass of the whole network.
evconv_status run_pass(evconv_net* net, const float* input, int builder_mode, PassKind pass) {
  hipStream_t s = net->stream;
  const int dense = pass != kPassStep;
  const bool reinit = pass == kPassReset || pass == kPassRefresh;  // sparsification residuals and steps restart
  const int int_mode = pass == kPassStep ? kIntStep : pass == kPassReset ? kIntReset : kIntRecompute;
  BuilderParams bp;
  bp.in = input; bp.x_prev = net->x_prev; bp.dx = net->dx; bp.occ = net->occ_in;
  bp.clear = net->occ_nodes; bp.n_clear = (int)net->L.n_occ_words;
  bp.g = net->L.gin; bp.mode = builder_mode;
  bp.st = net->st; bp.in_stride = net->in_stride;
  // per-launch timing (evconv_profile_begin): record r is an event pair around the launches of
  // prof_node[r]; -1 stands for the increment builder, n_nodes for the list compaction
  auto timed_begin = [&]() {
    const bool timed = net->prof && 2 * (net->prof_node.size() + 1) <= net->prof_ev.size();
    if (timed) (void)hipEventRecord(net->prof_ev[2 * net->prof_node.size()], s);
    return timed;
  };
  auto timed_end = [&](bool timed, int node) {
    if (!timed) return;
    (void)hipEventRecord(net->prof_ev[2 * net->prof_node.size() + 1], s);
    net->prof_node.push_back(node);
  };
  {
    const bool timed = timed_begin();
    launch_builder(bp, s);
    timed_end(timed, -1);
  }

  for (size_t i = 0; i < net->L.nodes.size(); ++i) {
    NodePlan& n = net->L.nodes[i];
    const evconv_node_desc& d = n.d;
    const float* a = d.in0 < 0 ? net->dx : net->L.nodes[d.in0].out;
    const uint64_t* occ_a = d.in0 < 0 ? net->occ_in : net->L.nodes[d.in0].occ;
    const bool two = d.op == EVCONV_OP_ADD || d.op == EVCONV_OP_CONCAT || d.op == EVCONV_OP_MUL;
    const float* bptr = two ? (d.in1 < 0 ? net->dx : net->L.nodes[d.in1].out) : nullptr;
    const uint64_t* occ_b = two ? (d.in1 < 0 ? net->occ_in : net->L.nodes[d.in1].occ) : nullptr;
    if (n.gather_fused_into >= 0) continue;  // exists only inside the consuming conv's gather
    if (n.kernel == kKernDelay) {
      const NodePlan& x = net->L.nodes[d.in0];  // not yet visited in this pass: holds the previous pass's results
      DelayParams p;
      p.src_out = x.out; p.occ_saved = n.occ_saved; p.z = n.z; p.out = n.out;
      p.occ_out = n.occ; p.occ_touched = n.touched; p.g = n.go;
      p.dense = dense; p.last_dense = net->last_dense; p.zero_state = net->zero_state;
      p.st = net->st;
      launch_delay(p, s);
      if (d.is_output) {
        IntegrateParams ip;
        ip.delta = n.out; ip.occ = n.occ; ip.y = n.y; ip.dy = n.dy; ip.g = n.go;
        ip.mode = int_mode;
        ip.st = net->st;
        launch_integrate(ip, s);
      }
      continue;
    }
    if (n.fused_into >= 0) {  // computed by the producing conv's epilogue
      if (d.op == EVCONV_OP_SPARSIFY && reinit && n.step_fixed < 0.0f)
        // refresh: k = t_p * RMS of the layer input, which the producer has just written in full
        launch_rms_step(a, (size_t)n.ga.c * n.ga.sites(), net->sparsify_tp, net->rms_partial, n.step, net->st, s);
      if (d.is_output) {
        IntegrateParams ip;
        ip.delta = n.out; ip.occ = n.occ; ip.y = n.y; ip.dy = n.dy; ip.g = n.go;
        ip.mode = int_mode;
        ip.st = net->st;
        launch_integrate(ip, s);
      }
      continue;
    }
    const bool timed = timed_begin();
    bool integrated = false;  // an output node whose kernel keeps the public tensors itself
    switch (n.kernel) {
      case kKernConvValu:
      case kKernConvNarrow:
      case kKernConvPointwise:
      case kKernConvMfmaSplit:
      case kKernConvMfmaBf16:
      case kKernConvMfmaF32: {
        ConvParams p;
        p.in = a; p.occ_in = occ_a; p.w = n.w; p.bias = n.bias; p.z = n.z; p.out = n.out;
        p.occ_out = n.occ; p.occ_touched = n.touched; p.gi = n.ga; p.go = n.go; p.c_out_pad = n.c_out_pad;
        p.k = d.kh; p.stride = d.stride; p.pad = d.pad; p.act = d.act; p.dense = dense;
        p.n_fused = n.n_fused;
        p.st = net->st;
        p.upsample = 0; p.lo_h = 0; p.lo_w = 0;
        p.y = nullptr; p.dy = nullptr; p.int_mode = 0;
        p.fold_list = n.fold_list; p.w_fold = n.w_fold; p.fold_k = n.fold_k; p.wg_swap = 0;
        p.fold_base[0] = n.fold_base[0]; p.fold_base[1] = n.fold_base[1];
        if (n.upsampled_from != -2) {
          // read the stored low-resolution tensor; p.gi stays the up-sampled geometry
          const int src = n.upsampled_from;
          p.in = src < 0 ? net->dx : net->L.nodes[src].out;
          p.occ_in = src < 0 ? net->occ_in : net->L.nodes[src].occ;
          const Geo& gl = src < 0 ? net->L.gin : net->L.nodes[src].go;
          p.upsample = 1; p.lo_h = gl.h; p.lo_w = gl.w;
        }
        p.sp = FusedSparsify{};
        if (n.fused_sp >= 0) {
          const NodePlan& sp = net->L.nodes[n.fused_sp];
          p.sp.delta = sp.z; p.sp.out = sp.out; p.sp.occ_out = sp.occ; p.sp.occ_touched = sp.touched; p.sp.step = sp.step;
        }
        for (int f = 0; f < kMaxFusedAdds; ++f) p.fused[f] = FusedAdd{};
        for (int f = 0; f < n.n_fused; ++f) {
          const NodePlan& a_node = net->L.nodes[n.fused_nodes[f]];
          // the ADD's other input: the one that is not the previous stage
          const int prev = f == 0 ? (int)i : n.fused_nodes[f - 1];
          const int other = a_node.d.in0 == prev ? a_node.d.in1 : a_node.d.in0;
          FusedAdd& fa = p.fused[f];
          fa.skip = other < 0 ? net->dx : net->L.nodes[other].out;
          fa.occ_skip = other < 0 ? net->occ_in : net->L.nodes[other].occ;
          fa.z = a_node.z; fa.out = a_node.out; fa.occ_out = a_node.occ; fa.occ_touched = a_node.touched;
          fa.act = a_node.d.act; fa.keeps_z = a_node.keeps_z; fa.structural = a_node.structural;
        }
        if (n.kernel == kKernConvPointwise && d.is_output && conv_pointwise_integrates(p)) {
          p.y = n.y; p.dy = n.dy;
          p.int_mode = int_mode;
          integrated = true;
        }
        if (n.kernel == kKernConvMfmaF32) launch_conv_mfma_f32(p, s);
        else if (n.kernel == kKernConvMfmaBf16) launch_conv_mfma_bf16(p, s);
        else if (n.kernel == kKernConvNarrow) launch_conv_narrow(p, s);
        else if (n.kernel == kKernConvPointwise) launch_conv_pointwise(p, s);
        else if (n.kernel == kKernConvMfmaSplit) launch_conv_mfma_split(p, s);
        else launch_conv_valu(p, s);
        break;
      }
      case kKernElementwise: {
        EwParams p;
        p.op = d.op == EVCONV_OP_ADD ? kEwAdd : d.op == EVCONV_OP_CONCAT ? kEwConcat : d.op == EVCONV_OP_MUL ? kEwMul :
               d.op == EVCONV_OP_UPSAMPLE_BILINEAR2X ? kEwUp2x : d.op == EVCONV_OP_SPARSIFY ? kEwSparsify : kEwAct;
        p.step = n.step;
        p.st = net->st;
        if (d.op == EVCONV_OP_SPARSIFY && reinit && n.step_fixed < 0.0f)
          // refresh: k = t_p * RMS of the layer input, which the producer has just written in full
          launch_rms_step(a, (size_t)n.ga.c * n.ga.sites(), net->sparsify_tp, net->rms_partial, n.step, net->st, s);
        p.act = d.act; p.dense = dense; p.keeps_z = n.keeps_z; p.structural = n.structural;
        p.ga = n.ga; p.gb = n.gb; p.go = n.go; p.a = a; p.occ_a = occ_a; p.b = bptr; p.occ_b = occ_b;
        if (d.op == EVCONV_OP_CONCAT && n.upsampled_from != -2) {
          // the first operand is an up-sampling that is never stored: read its stored source
          const int src = n.upsampled_from;
          p.op = kEwConcatUp;
          p.a = src < 0 ? net->dx : net->L.nodes[src].out;
          p.occ_a = src < 0 ? net->occ_in : net->L.nodes[src].occ;
          p.ga = src < 0 ? net->L.gin : net->L.nodes[src].go;
        }
        p.z = n.z; p.z2 = n.z2; p.out = n.out; p.occ_out = n.occ; p.occ_touched = n.touched;
        p.k = 1; p.stride = 1; p.pad = 0;
        launch_elementwise(p, s);
        break;
      }
      case kKernPool: {
        EwParams p;
        p.st = net->st; p.z2 = nullptr; p.step = nullptr;
        p.act = kActNone; p.dense = dense; p.keeps_z = 0; p.structural = 0;
        p.ga = n.ga; p.gb = n.ga; p.a = a; p.occ_a = occ_a; p.b = nullptr; p.occ_b = nullptr;
        p.out = nullptr; p.occ_out = nullptr; p.occ_touched = nullptr;
        p.k = d.kh; p.stride = d.stride; p.pad = d.pad;
        p.op = kEwPoolAcc; p.go = n.ga; p.z = n.pool_in;  // a_acc += x_inc on S_in
        launch_elementwise(p, s);
        p.op = kEwPoolMax; p.go = n.go; p.a = n.pool_in; p.z = n.z; p.out = n.out;
        p.occ_out = n.occ; p.occ_touched = n.touched;
        launch_elementwise(p, s);
        break;
      }
      case kKernGap: {
        GapParams p;
        p.a = a; p.occ_a = occ_a; p.ga = n.ga; p.z = n.z; p.out = n.out; p.occ_out = n.occ;
        p.occ_touched = n.touched; p.act = d.act; p.dense = dense;
        p.st = net->st;
        launch_gap(p, s);
        break;
      }
    }
    timed_end(timed, (int)i);
    if (d.is_output && !integrated) {
      IntegrateParams ip;
      ip.delta = n.out; ip.occ = n.occ; ip.y = n.y; ip.dy = n.dy; ip.g = n.go;
      ip.mode = int_mode;
      ip.st = net->st;
      launch_integrate(ip, s);
    }
  }
  // recurrent state: keep the delayed nodes' active sets for the next pass (the occupancy words
  // are cleared when it starts)
  for (size_t i = 0; i < net->L.nodes.size(); ++i) {
    const NodePlan& n = net->L.nodes[i];
    if (n.kernel == kKernDelay) launch_copy_u64(n.occ_saved, net->L.nodes[n.d.in0].occ, (size_t)n.go.tiles(), net->st, s);
  }
  net->last_dense = dense != 0;
  if (pass == kPassReset) launch_fill_u64(net->occ_nodes, net->L.n_occ_words, 0, net->st, s);
  if (pass == kPassRefresh) {
    // the nodes' buffers hold values, not increments: every set is emptied, except the active sets of
    // the output nodes, whose dy = y(n) - y(n-1) is a genuine increment at every site
    size_t from = 0;
    for (size_t i = 0; i <= net->L.nodes.size(); ++i) {
      const bool last = i == net->L.nodes.size();
      if (!last && !net->L.nodes[i].d.is_output) continue;
      const size_t to = last ? net->L.n_occ_words : (size_t)(net->L.nodes[i].occ - net->occ_nodes);
      if (to > from) launch_fill_u64(net->occ_nodes + from, to - from, 0, net->st, s);
      if (!last) from = to + (size_t)net->L.nodes[i].go.tiles();  // skip the S words, clear the T words behind them
    }
  }
  {
    const bool timed = timed_begin();
    launch_build_lists(net->sets_dev, (int)net->L.nodes.size() + 1, net->L.max_ty, net->st, s);
    timed_end(timed, (int)net->L.nodes.size());
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(net, e, "kernel launch");
  return EVCONV_OK;
}

void fill_outputs(evconv_net* net, evconv_out* out) {
  if (!out) return;
  for (size_t j = 0; j < net->outputs.size(); ++j) {
    const NodePlan& n = net->L.nodes[net->outputs[j]];
    out[j].node = net->outputs[j];
    out[j].c = n.go.c; out[j].h = n.go.h; out[j].w = n.go.w;
    out[j].y = n.y; out[j].dy = n.dy; out[j].dy_idx = n.idx; out[j].dy_count = n.count;
  }
}

// Weight folding for a conv (k x k, pad k/2, stride 1) that reads through a bilinear x2
// up-sampling (half-pixel centres: row 2q of the up-sampled tensor is 0.75 * stored row q + 0.25 *
// row q - 1, row 2q + 1 is 0.75 * row q + 0.25 * row q + 1).  Both are linear (Eq.9), so for
// outputs of one parity the composition is a conv on the stored tensor with kf < k taps per
// dimension.  That holds where the window meets neither the clamped first / last up-sampled row
// nor the conv's zero padding: stored sites `edge` or more away from the border.  Tiles of stored
// sites made of such sites only are computed per phase with the folded weights; the up-sampled
// tiles over all other stored tiles go through the interpolating gather.  Writes the four weight
// sets and the tile list into the workspace.  `lo` is the stored tensor's geometry.
hipError_t prepare_fold(evconv_net* net, NodePlan& n, const void* weights, const Geo& lo) {
  const int k = n.d.kh, pad = n.d.pad, ci_n = n.d.c_in, co_n = n.d.c_out, cop = n.c_out_pad;
  int base[2], main_row[2][8], other_row[2][8], kf = 0;
  for (int par = 0; par < 2; ++par) {
    int first = 1 << 20, last = -(1 << 20);
    for (int ky = 0; ky < k; ++ky) {
      const int r = par + ky - pad;                       // up-sampled row relative to 2 * (stored row)
      const int q = r >= 0 ? r / 2 : -((1 - r) / 2);      // floor(r / 2)
      main_row[par][ky] = q;
      other_row[par][ky] = (r - 2 * q) ? q + 1 : q - 1;
      first = std::min(first, std::min(main_row[par][ky], other_row[par][ky]));
      last = std::max(last, std::max(main_row[par][ky], other_row[par][ky]));
    }
    base[par] = first;
    kf = std::max(kf, last - first + 1);
  }
  const int edge = (pad + 2) / 2;
  auto interior = [&](int t, int n_sites) { return 8 * t >= edge && 8 * t + 7 <= n_sites - 1 - edge; };
  std::vector<int> list;
  for (int ty = 0; ty < n.go.ty; ++ty)
    for (int tx = 0; tx < n.go.tx; ++tx)
      if (!(interior(ty / 2, lo.h) && interior(tx / 2, lo.w))) list.push_back(ty * n.go.tx + tx);
  // (the border tiles' workgroups run longest: they come first; interleaving them with the folded
  // ones measured 3.5 % slower)
  if ((int)list.size() == n.go.tiles()) return hipSuccess;  // nothing away from the border: no folding
  // Consecutive workgroups go to the chip's 8 XCDs in turn, each with an L2 of its own.  With the
  // four phases of a tile next to each other an XCD runs one phase only and so reads one of the
  // four weight sets (measured: placing a tile's phases on one XCD instead, to share the patch,
  // raises the HBM fetch of the launches by 12 %: the weights outweigh the patches).
  for (int ty = 0; ty < lo.ty; ++ty)
    for (int tx = 0; tx < lo.tx; ++tx)
      if (interior(ty, lo.h) && interior(tx, lo.w))
        for (int ph = 0; ph < 4; ++ph) list.push_back(-(1 + 4 * (ty * lo.tx + tx) + ph));
  if ((int)list.size() != n.go.tiles() || kf != 4) return hipSuccess;  // (room was reserved for 4 x 4 taps)

  const float* src = (const float*)((const char*)weights + n.d.weight_off);
  const int taps = kf * kf;
  std::vector<double> folded((size_t)4 * taps * ci_n * co_n, 0.0);
  for (int py = 0; py < 2; ++py)
    for (int px = 0; px < 2; ++px)
      for (int ky = 0; ky < k; ++ky)
        for (int kx = 0; kx < k; ++kx)
          for (int sy = 0; sy < 2; ++sy)
            for (int sx = 0; sx < 2; ++sx) {
              const int ty = (sy ? other_row[py][ky] : main_row[py][ky]) - base[py];
              const int tx = (sx ? other_row[px][kx] : main_row[px][kx]) - base[px];
              const double coef = (sy ? 0.25 : 0.75) * (sx ? 0.25 : 0.75);
              double* dst = &folded[((size_t)(py * 2 + px) * taps + ty * kf + tx) * ci_n * co_n];
              for (int co = 0; co < co_n; ++co)
                for (int ci = 0; ci < ci_n; ++ci)
                  dst[(size_t)ci * co_n + co] += coef * (double)src[((size_t)co * ci_n + ci) * k * k + ky * k + kx];
            }
  const int ci_p = (ci_n + 31) / 32 * 32;
  const size_t set = (size_t)taps * ci_p * cop;  // fp32 words per phase (two bf16 planes in split mode)
  std::vector<float> staging(4 * set, 0.0f);
  for (int ph = 0; ph < 4; ++ph)
    for (int t = 0; t < taps; ++t)
      for (int ci = 0; ci < ci_n; ++ci)
        for (int co = 0; co < co_n; ++co) {
          const float w = (float)folded[(((size_t)ph * taps + t) * ci_n + ci) * co_n + co];
          if (n.kernel == kKernConvMfmaSplit) {
            uint16_t* h16 = (uint16_t*)(staging.data() + ph * set);
            const size_t at = (((size_t)t * (ci_p / 8) + ci / 8) * cop + co) * 8 + (ci & 7);
            const uint16_t hi = to_bf16(w);
            const uint32_t hu = (uint32_t)hi << 16;
            float hf;
            memcpy(&hf, &hu, 4);
            h16[at] = hi;
            h16[set + at] = to_bf16(w - hf);  // the low plane follows the high plane: `set` bf16 each
          } else {
            staging[ph * set + (((size_t)t * (ci_p / 4) + ci / 4) * cop + co) * 4 + (ci & 3)] = w;
          }
        }
  n.w_fold = net->ws + n.off_w_fold;
  n.fold_list = (int*)(net->ws + n.off_fold_list);
  n.fold_k = kf;
  n.fold_base[0] = base[0];
  n.fold_base[1] = base[1];
  hipError_t e = hipMemcpy(n.w_fold, staging.data(), staging.size() * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(n.fold_list, list.data(), list.size() * 4, hipMemcpyHostToDevice);
  return e;
}

}  // namespace

extern "C" {

evconv_status evconv_query_workspace(const evconv_net_desc* desc, size_t* bytes) {
  if (!bytes) return EVCONV_ERR_INVALID_ARG;
  Layout L;
  evconv_status st = make_layout(desc, 0, false, &L, &g_create_error);
  if (st != EVCONV_OK) return st;
  *bytes = L.total;
  return EVCONV_OK;
}

}  // extern "C"

namespace {
evconv_status create_impl(const evconv_net_desc* desc, const void* weights, size_t weight_bytes,
                          void* workspace, size_t workspace_bytes, void* hip_stream, evconv_net** out) {
  if (!out || !workspace || (!weights && weight_bytes)) {
    g_create_error = "null argument";
    return EVCONV_ERR_INVALID_ARG;
  }
  evconv_net* net = new evconv_net();
  evconv_status st = make_layout(desc, weight_bytes, true, &net->L, &g_create_error);
  if (st != EVCONV_OK) { delete net; return st; }
  if (((uintptr_t)workspace & 255) || workspace_bytes < net->L.total) {
    g_create_error = "workspace too small or not 256-byte aligned";
    delete net;
    return EVCONV_ERR_WORKSPACE;
  }
  Layout& L = net->L;
  net->ws = (char*)workspace;
  net->stream = (hipStream_t)hip_stream;
  net->desc_nodes.assign(desc->nodes, desc->nodes + desc->n_nodes);
  char* ws = net->ws;
  net->x_prev = (float*)(ws + L.off_x_prev);
  net->dx = (float*)(ws + L.off_dx);
  net->occ_in = (uint64_t*)(ws + L.off_occ_in);
  net->idx_in = (int32_t*)(ws + L.off_idx_in);
  net->count_in = (int32_t*)(ws + L.off_count_in);
  net->bitmap_in = (uint64_t*)(ws + L.off_bitmap_in);
  net->occ_nodes = (uint64_t*)(ws + L.off_occ_nodes);
  net->sets_dev = (SetDesc*)(ws + L.off_sets);
  net->rms_partial = (float*)(ws + L.off_rms);
  net->sparsify_tp = desc->sparsify_tp;
  net->flags = desc->flags;
  net->st = Streams{L.stride, L.n_streams};
  net->in_stride = (size_t)L.gin.c * L.gin.sites() * sizeof(float);

  // (the uploads below are blocking copies that are not ordered with a non-blocking caller stream:
  // the clearing has to be complete before the first of them)
  hipError_t e = hipMemsetAsync(ws, 0, L.total, net->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(net->stream);
  if (e != hipSuccess) { g_create_error = std::string("clearing the workspace: ") + hipGetErrorString(e); delete net; return EVCONV_ERR_HIP; }

  std::vector<SetDesc> sets(L.nodes.size() + 1);
  sets[0] = SetDesc{net->occ_in, net->idx_in, net->count_in, net->bitmap_in, L.gin.h, L.gin.w, L.gin.tx, L.gin.ty};
  std::vector<float> staging;
  for (size_t i = 0; i < L.nodes.size(); ++i) {
    NodePlan& n = L.nodes[i];
    const size_t elems = (size_t)n.go.c * n.go.sites();
    (void)elems;
    n.z = (n.keeps_z || n.d.op == EVCONV_OP_MAXPOOL) ? (float*)(ws + n.off_z) : nullptr;
    if (n.d.op == EVCONV_OP_SPARSIFY) {
      n.step = (float*)(ws + n.off_step);
      if (n.d.weight_off < 0 && desc->sparsify_tp > 0.0f) net->has_sparsify = true;
      if (n.d.weight_off >= 0) {
        memcpy(&n.step_fixed, (const char*)weights + n.d.weight_off, 4);
        if (!(n.step_fixed >= 0.0f)) { g_create_error = "negative sparsification step"; delete net; return EVCONV_ERR_BAD_DESC; }
        if (n.step_fixed > 0.0f) net->has_sparsify = true;
        for (int sidx = 0; sidx < L.n_streams && e == hipSuccess; ++sidx)
          e = hipMemcpy((char*)n.step + (size_t)sidx * L.stride, &n.step_fixed, 4, hipMemcpyHostToDevice);
        if (e != hipSuccess) { g_create_error = std::string("upload: ") + hipGetErrorString(e); delete net; return EVCONV_ERR_HIP; }
      }
    }
    n.pool_in = n.d.op == EVCONV_OP_MAXPOOL ? (float*)(ws + n.off_pool) : nullptr;
    n.z2 = n.d.op == EVCONV_OP_MUL ? (float*)(ws + n.off_z2) : nullptr;
    n.occ_saved = n.d.op == EVCONV_OP_DELAY ? (uint64_t*)(ws + n.off_occ_saved) : nullptr;
    n.out = (float*)(ws + n.off_out);
    n.occ = (uint64_t*)(ws + n.off_occ);
    n.touched = (uint64_t*)(ws + n.off_touched);
    n.idx = (int32_t*)(ws + n.off_idx);
    n.count = (int32_t*)(ws + n.off_count);
    n.bitmap = (uint64_t*)(ws + n.off_bitmap);
    if (n.d.is_output) {
      n.y = (float*)(ws + n.off_y);
      n.dy = (float*)(ws + n.off_dy);
      net->outputs.push_back((int)i);
    }
    sets[i + 1] = SetDesc{n.occ, n.idx, n.count, n.bitmap, n.go.h, n.go.w, n.go.tx, n.go.ty};
    if (n.d.op == EVCONV_OP_CONV2D || n.d.op == EVCONV_OP_LINEAR) {
      const int k = n.d.kh, ci_n = n.d.c_in, co_n = n.d.c_out, cop = n.c_out_pad;
      ConvParams probe;
      probe.gi = n.ga; probe.go = n.go; probe.k = k; probe.stride = n.d.stride; probe.c_out_pad = cop;
      probe.n_fused = 0; probe.pad = n.d.pad; probe.st = Streams{L.stride, L.n_streams};
      const bool force_valu = (net->flags & EVCONV_FLAG_FORCE_VALU) != 0;
      if (!force_valu && n.d.wdtype == EVCONV_F32 && conv_mfma_f32_supported(probe)) n.kernel = kKernConvMfmaF32;
      if (!force_valu && n.d.wdtype == EVCONV_BF16 && conv_mfma_bf16_supported(probe)) n.kernel = kKernConvMfmaBf16;
      if (!force_valu && n.d.wdtype == EVCONV_F32_SPLIT && conv_mfma_split_supported(probe)) n.kernel = kKernConvMfmaSplit;
      if (!force_valu && n.kernel == kKernConvValu && conv_narrow_supported(probe)) n.kernel = kKernConvNarrow;
      if (!force_valu && conv_pointwise_supported(probe)) n.kernel = kKernConvPointwise;
      const float* src = (const float*)((const char*)weights + n.d.weight_off);
      staging.assign(((size_t)k * k * ((ci_n + 63) / 64 * 64) + 16) * cop, 0.0f);
      const int ci_p = conv_mfma_padded_cin(probe);  // matrix-core kinds: channels padded with zero rows
      if (n.kernel == kKernConvPointwise) {
        // 1 x 1 taps: [c_out][c_in] as supplied; bf16-declared weights are rounded and widened again
        staging.resize((size_t)co_n * ci_n);
        for (size_t e = 0; e < staging.size(); ++e) {
          float w = src[e];
          if (n.d.wdtype == EVCONV_BF16) {
            const uint32_t u = (uint32_t)to_bf16(w) << 16;
            memcpy(&w, &u, 4);
          }
          staging[e] = w;
        }
      } else if (n.kernel == kKernConvNarrow) {
        // flattened contraction k = tap * c_in + ci, laid out per matrix-core lane, zeros beyond
        // taps * c_in and beyond c_out; bf16-declared weights are rounded to bf16 and widened again
        staging.assign(conv_narrow_weight_floats(cop), 0.0f);
        for (int co = 0; co < co_n; ++co)
          for (int ci = 0; ci < ci_n; ++ci)
            for (int t = 0; t < k * k; ++t) {
              float w = src[((size_t)co * ci_n + ci) * k * k + t];
              if (n.d.wdtype == EVCONV_BF16) {
                const uint32_t u = (uint32_t)to_bf16(w) << 16;
                memcpy(&w, &u, 4);
              }
              staging[conv_narrow_weight_index(t * ci_n + ci, co)] = w;
            }
      } else if (n.kernel == kKernConvMfmaSplit) {
        // two bf16 planes [tap][c_in/8][c_out][8]: hi = bf16(w), then lo = bf16(w - hi)
        uint16_t* h16 = (uint16_t*)staging.data();
        const size_t plane = (size_t)k * k * ci_p * cop;
        for (int co = 0; co < co_n; ++co)
          for (int ci = 0; ci < ci_n; ++ci)
            for (int t = 0; t < k * k; ++t) {
              const float w = src[((size_t)co * ci_n + ci) * k * k + t];
              const uint16_t hi = to_bf16(w);
              float hf;
              const uint32_t hu = (uint32_t)hi << 16;
              memcpy(&hf, &hu, 4);
              const size_t at = (((size_t)t * (ci_p / 8) + ci / 8) * cop + co) * 8 + (ci & 7);
              h16[at] = hi;
              h16[plane + at] = to_bf16(w - hf);
            }
      } else if (n.kernel == kKernConvMfmaBf16) {
        // bf16 matrix-core layout [tap][c_in/8][c_out][8]: a lane's 8 input channels are 16 bytes
        uint16_t* h16 = (uint16_t*)staging.data();
        for (int co = 0; co < co_n; ++co)
          for (int ci = 0; ci < ci_n; ++ci)
            for (int t = 0; t < k * k; ++t)
              h16[(((size_t)t * (ci_p / 8) + ci / 8) * cop + co) * 8 + (ci & 7)] =
                  to_bf16(src[((size_t)co * ci_n + ci) * k * k + t]);
      } else if (n.kernel == kKernConvMfmaF32) {
        // matrix-core layout [tap][c_in/4][c_out][4]: a lane's 4 input channels are 16 bytes
        for (int co = 0; co < co_n; ++co)
          for (int ci = 0; ci < ci_n; ++ci)
            for (int t = 0; t < k * k; ++t)
              staging[(((size_t)t * (ci_p / 4) + ci / 4) * cop + co) * 4 + (ci & 3)] =
                  src[((size_t)co * ci_n + ci) * k * k + t];
      } else {
        // vector-ALU layout [tap][c_in][c_out_pad] (zero padded output channels)
        for (int co = 0; co < co_n; ++co)
          for (int ci = 0; ci < ci_n; ++ci)
            for (int t = 0; t < k * k; ++t)
              staging[((size_t)t * ci_n + ci) * cop + co] = src[((size_t)co * ci_n + ci) * k * k + t];
      }
      n.w = ws + n.off_w;
      e = hipMemcpyAsync(n.w, staging.data(), staging.size() * 4, hipMemcpyHostToDevice, net->stream);
      if (e == hipSuccess) e = hipStreamSynchronize(net->stream);  // staging is reused
      if (e == hipSuccess && n.d.bias_off >= 0) {
        n.bias = (float*)(ws + n.off_bias);
        e = hipMemcpy(n.bias, (const char*)weights + n.d.bias_off, (size_t)co_n * 4, hipMemcpyHostToDevice);
      }
      if (e != hipSuccess) { g_create_error = std::string("weight upload: ") + hipGetErrorString(e); delete net; return EVCONV_ERR_HIP; }
    }
  }
  e = hipMemcpyAsync(net->sets_dev, sets.data(), sets.size() * sizeof(SetDesc), hipMemcpyHostToDevice, net->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(net->stream);
  if (e != hipSuccess) { g_create_error = std::string("upload: ") + hipGetErrorString(e); delete net; return EVCONV_ERR_HIP; }
  if (net->outputs.empty()) { g_create_error = "no output node"; delete net; return EVCONV_ERR_BAD_DESC; }
  // Fold ADD nodes into the epilogue of the matrix-core conv that produces their later input
  // (residual add + activation, skip adds).  Every buffer of the ADD node is still written.
  const bool fuse = !(net->flags & EVCONV_FLAG_NO_FUSION);
  if (fuse) {
    for (size_t i = 0; i < L.nodes.size(); ++i) {
      NodePlan& a_node = L.nodes[i];
      if (a_node.d.op != EVCONV_OP_ADD) continue;
      const int later = a_node.d.in0 > a_node.d.in1 ? a_node.d.in0 : a_node.d.in1;
      const int other = a_node.d.in0 > a_node.d.in1 ? a_node.d.in1 : a_node.d.in0;
      if (later < 0 || later == other) continue;
      const int host = L.nodes[later].fused_into >= 0 ? L.nodes[later].fused_into : later;
      NodePlan& c_node = L.nodes[host];
      if ((c_node.kernel != kKernConvMfmaF32 && c_node.kernel != kKernConvMfmaBf16 &&
           c_node.kernel != kKernConvMfmaSplit) ||
          c_node.n_fused >= kMaxFusedAdds) continue;
      if (host != later && c_node.fused_nodes[c_node.n_fused - 1] != later) continue;  // chain must be contiguous
      if (other >= host) continue;  // the other input must exist before the conv runs
      // A DELAY node between the conv and the ADD that delays this ADD reads the ADD's buffers as
      // the previous step left them; computed in the conv's epilogue they would already hold
      // this step's values.
      bool delayed_between = false;
      for (size_t dn = (size_t)host + 1; dn < i; ++dn)
        if (L.nodes[dn].d.op == EVCONV_OP_DELAY && L.nodes[dn].d.in0 == (int)i) delayed_between = true;
      if (delayed_between) continue;
      c_node.fused_nodes[c_node.n_fused++] = (int)i;
      a_node.fused_into = host;
    }
  }
  // Fold a sparsification layer into the epilogue of the matrix-core conv that produces its input,
  // directly or through the last ADD folded into that conv: the layer then reads the increment
  // where it is made (no launch, no re-read).  One layer per conv; every buffer of the layer is
  // still written.
  if (fuse) {
    for (size_t i = 0; i < L.nodes.size(); ++i) {
      NodePlan& s_node = L.nodes[i];
      if (s_node.d.op != EVCONV_OP_SPARSIFY || s_node.d.in0 < 0 || s_node.d.is_output) continue;
      const NodePlan& x = L.nodes[s_node.d.in0];
      int host = -1;
      if (x.fused_into >= 0) {
        const NodePlan& h = L.nodes[x.fused_into];
        if (x.d.op == EVCONV_OP_ADD && h.n_fused > 0 && h.fused_nodes[h.n_fused - 1] == s_node.d.in0) host = x.fused_into;
      } else if (x.n_fused == 0 && (x.kernel == kKernConvMfmaF32 || x.kernel == kKernConvMfmaBf16 || x.kernel == kKernConvMfmaSplit)) {
        host = s_node.d.in0;
      }
      if (host < 0 || L.nodes[host].fused_sp >= 0) continue;
      bool delayed_between = false;  // (a DELAY of this layer placed before it must see last step's buffers)
      for (size_t dn = (size_t)host + 1; dn < i; ++dn)
        if (L.nodes[dn].d.op == EVCONV_OP_DELAY && L.nodes[dn].d.in0 == (int)i) delayed_between = true;
      if (delayed_between) continue;
      L.nodes[host].fused_sp = (int)i;
      s_node.fused_into = host;
    }
  }
  // Fold a bilinear x2 up-sampling into the gather of the matrix-core conv that is its only
  // consumer: the up-sampled tensor is then never written (its node keeps no state).
  if (fuse) {
    std::vector<int> n_consumers(L.nodes.size(), 0);
    for (size_t i = 0; i < L.nodes.size(); ++i) {
      const evconv_node_desc& d = L.nodes[i].d;
      if (d.in0 >= 0) ++n_consumers[d.in0];
      const bool two = d.op == EVCONV_OP_ADD || d.op == EVCONV_OP_CONCAT || d.op == EVCONV_OP_MUL;
      if (two && d.in1 >= 0 && d.in1 != d.in0) ++n_consumers[d.in1];
    }
    for (size_t i = 0; i < L.nodes.size(); ++i) {
      NodePlan& c_node = L.nodes[i];
      if (c_node.d.op != EVCONV_OP_CONV2D || c_node.d.in0 < 0) continue;
      NodePlan& u_node = L.nodes[c_node.d.in0];
      if (u_node.d.op != EVCONV_OP_UPSAMPLE_BILINEAR2X || u_node.d.act != EVCONV_ACT_NONE || u_node.d.is_output ||
          n_consumers[c_node.d.in0] != 1 || u_node.fused_into >= 0) continue;
      if (c_node.kernel != kKernConvMfmaF32 && c_node.kernel != kKernConvMfmaBf16 && c_node.kernel != kKernConvMfmaSplit)
        continue;
      ConvParams probe;
      probe.gi = c_node.ga; probe.go = c_node.go; probe.k = c_node.d.kh; probe.stride = c_node.d.stride;
      probe.c_out_pad = c_node.c_out_pad; probe.n_fused = 0; probe.pad = c_node.d.pad;
      probe.st = Streams{L.stride, L.n_streams};
      if (!conv_mfma_upsample_supported(probe)) continue;
      u_node.gather_fused_into = (int)i;
      c_node.upsampled_from = u_node.d.in0;
      // away from the image border the up-sampling goes into the weights instead (fp32 products only:
      // bf16-declared weights would be rounded a second time)
      if (c_node.off_fold_list && c_node.kernel != kKernConvMfmaBf16 && !(net->flags & EVCONV_FLAG_NO_FOLD)) {
        const Geo& lo = u_node.d.in0 < 0 ? L.gin : L.nodes[u_node.d.in0].go;
        e = prepare_fold(net, c_node, weights, lo);
        if (e != hipSuccess) { g_create_error = std::string("folded weights upload: ") + hipGetErrorString(e); delete net; return EVCONV_ERR_HIP; }
      }
    }
    // the same for a CONCAT whose first operand is an up-sampling nobody else reads: one kernel
    // interpolates that operand's channels and copies the other's
    for (size_t i = 0; i < L.nodes.size(); ++i) {
      NodePlan& c_node = L.nodes[i];
      if (c_node.d.op != EVCONV_OP_CONCAT || c_node.d.in0 < 0 || c_node.d.in0 == c_node.d.in1) continue;
      NodePlan& u_node = L.nodes[c_node.d.in0];
      if (u_node.d.op != EVCONV_OP_UPSAMPLE_BILINEAR2X || u_node.d.act != EVCONV_ACT_NONE || u_node.d.is_output ||
          n_consumers[c_node.d.in0] != 1 || u_node.fused_into >= 0 || u_node.gather_fused_into >= 0) continue;
      u_node.gather_fused_into = (int)i;
      c_node.upsampled_from = u_node.d.in0;
    }
  }
  *out = net;
  return EVCONV_OK;
}
}  // namespace

extern "C" {

evconv_status evconv_create(const evconv_net_desc* desc, const void* weights, size_t weight_bytes,
                            void* workspace, size_t workspace_bytes, void* hip_stream, evconv_net** out) {
  return create_impl(desc, weights, weight_bytes, workspace, workspace_bytes, hip_stream, out);
}

evconv_status evconv_create_static(const evconv_net_desc* desc, const void* weights, size_t weight_bytes,
                                   void* hip_stream, evconv_net** out) {
  if (!out) { g_create_error = "null argument"; return EVCONV_ERR_INVALID_ARG; }
  Layout L;
  evconv_status st = make_layout(desc, weight_bytes, true, &L, &g_create_error);
  if (st != EVCONV_OK) return st;
  if (L.total > (size_t)EVCONV_STATIC_WORKSPACE_BYTES) {
    g_create_error = "this description needs " + std::to_string(L.total) + " bytes of workspace, the static workspace holds " +
                     std::to_string((size_t)EVCONV_STATIC_WORKSPACE_BYTES);
    return EVCONV_ERR_WORKSPACE;
  }
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    g_create_error = e != hipSuccess ? std::string("hipGetDevice: ") + hipGetErrorString(e) : "device index out of range";
    return EVCONV_ERR_HIP;
  }
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (g_static_owner[dev]) {
    g_create_error = "the static workspace of this device is in use by a net that has not been destroyed";
    return EVCONV_ERR_STATE;
  }
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      g_create_error = std::string("hipGetSymbolAddress: ") + hipGetErrorString(e);
      return EVCONV_ERR_HIP;
    }
    g_scratch_ptr[dev] = ptr;
  }
  // (create_impl clears the part of the array it lays the net out in: the array keeps whatever the
  // previous net left there)
  evconv_net* net = nullptr;
  st = create_impl(desc, weights, weight_bytes, g_scratch_ptr[dev], (size_t)EVCONV_STATIC_WORKSPACE_BYTES, hip_stream, &net);
  if (st != EVCONV_OK) return st;
  net->static_device = dev;
  g_static_owner[dev] = net;
  *out = net;
  return EVCONV_OK;
}

int32_t evconv_num_outputs(const evconv_net* net) { return net ? (int32_t)net->outputs.size() : 0; }

evconv_status evconv_reset(evconv_net* net, const float* x0, evconv_out* out) {
  if (!net) return EVCONV_ERR_INVALID_ARG;
  if (!x0) { net->err = "null x0"; return EVCONV_ERR_INVALID_ARG; }
  net->zero_state = true;
  evconv_status st = run_pass(net, x0, kBuildReset, kPassReset);
  net->zero_state = false;
  if (st != EVCONV_OK) return st;
  net->has_state = true;
  net->since_refresh = 0;
  fill_outputs(net, out);
  return EVCONV_OK;
}

static evconv_status step_common(evconv_net* net, const float* in, int builder_mode, evconv_out* out) {
  if (!net) return EVCONV_ERR_INVALID_ARG;
  if (!in) { net->err = "null input"; return EVCONV_ERR_INVALID_ARG; }
  if (!net->has_state) { net->err = "step before reset"; return EVCONV_ERR_STATE; }
  evconv_status st;
  const bool refresh = net->refresh_period > 0 && net->since_refresh + 1 >= net->refresh_period;
  int mode = net->mode;
  hipEvent_t ev_after = nullptr;
  if (mode == EVCONV_MODE_AUTO) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    (void)hipStreamIsCapturing(net->stream, &cap);
    if (net->has_sparsify || cap != hipStreamCaptureStatusNone || refresh) {
      mode = net->has_sparsify ? EVCONV_MODE_INCREMENTAL : net->auto_choice;
      if (refresh && net->auto_phase < 2) net->auto_count = 0;  // a window holding a refresh is timed again
    } else {
      if (net->auto_pending && hipEventQuery(net->auto_ev[3]) == hipSuccess) {
        float t_inc = 0.f, t_dense = 0.f;
        if (hipEventElapsedTime(&t_inc, net->auto_ev[0], net->auto_ev[1]) == hipSuccess &&
            hipEventElapsedTime(&t_dense, net->auto_ev[2], net->auto_ev[3]) == hipSuccess)
          net->auto_choice = t_dense < t_inc ? EVCONV_MODE_DENSE_RECOMPUTE : EVCONV_MODE_INCREMENTAL;
        net->auto_pending = false;
      }
      (void)hipGetLastError();  // (hipErrorNotReady of the query is not an error of this net)
      if (net->auto_phase == 2 && net->auto_count >= kAutoHold && !net->auto_pending) {
        net->auto_phase = 0;
        net->auto_count = 0;
      }
      mode = net->auto_phase == 0 ? EVCONV_MODE_INCREMENTAL : net->auto_phase == 1 ? EVCONV_MODE_DENSE_RECOMPUTE : net->auto_choice;
      if (net->auto_phase < 2) {
        if (net->auto_count == 0) (void)hipEventRecord(net->auto_ev[2 * net->auto_phase], net->stream);
        if (net->auto_count == kAutoProbe - 1) ev_after = net->auto_ev[2 * net->auto_phase + 1];
      }
      if (++net->auto_count >= kAutoProbe && net->auto_phase < 2) {
        if (net->auto_phase == 1) net->auto_pending = true;
        ++net->auto_phase;
        net->auto_count = 0;
      }
    }
  }
  if (refresh) {
    // "Drift Errors": every N-th step is a regular forward pass of x(n) that re-initialises every
    // accumulated tensor (and the sparsification residuals and step sizes)
    st = run_pass(net, in, builder_mode == kBuildFrame ? kBuildReset : kBuildIncrementDense, kPassRefresh);
    net->since_refresh = 0;
  } else if (mode == EVCONV_MODE_DENSE_RECOMPUTE) {
    // regular forward pass of x(n): the builder first folds the input into x_prev (and, for a
    // supplied increment, adds it), then the dense pass reads the updated frame
    st = run_pass(net, in, builder_mode == kBuildFrame ? kBuildReset : kBuildIncrementDense, kPassRecompute);
  } else {
    st = run_pass(net, in, builder_mode, kPassStep);
    ++net->since_refresh;
  }
  if (ev_after) (void)hipEventRecord(ev_after, net->stream);
  if (st != EVCONV_OK) return st;
  fill_outputs(net, out);
  return EVCONV_OK;
}

evconv_status evconv_step(evconv_net* net, const float* increment, evconv_out* out) {
  return step_common(net, increment, kBuildIncrement, out);
}

evconv_status evconv_step_frame(evconv_net* net, const float* x_t, evconv_out* out) {
  return step_common(net, x_t, kBuildFrame, out);
}

evconv_status evconv_destroy(evconv_net* net) {
  if (!net) return EVCONV_OK;
  (void)hipStreamSynchronize(net->stream);
  for (hipEvent_t e : net->prof_ev) (void)hipEventDestroy(e);
  for (hipEvent_t e : net->auto_ev)
    if (e) (void)hipEventDestroy(e);
  if (net->static_device >= 0) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (g_static_owner[net->static_device] == net) g_static_owner[net->static_device] = nullptr;
  }
  delete net;
  return EVCONV_OK;
}

evconv_status evconv_set_mode(evconv_net* net, int32_t mode) {
  if (!net) return EVCONV_ERR_INVALID_ARG;
  if (mode != EVCONV_MODE_INCREMENTAL && mode != EVCONV_MODE_DENSE_RECOMPUTE && mode != EVCONV_MODE_AUTO) {
    net->err = "bad mode";
    return EVCONV_ERR_INVALID_ARG;
  }
  if (mode == EVCONV_MODE_AUTO) {
    for (hipEvent_t& e : net->auto_ev)
      if (!e) {
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) return hip_fail(net, err, "hipEventCreate");
      }
    net->auto_phase = 0;
    net->auto_count = 0;
    net->auto_pending = false;
    net->auto_choice = EVCONV_MODE_INCREMENTAL;
  }
  net->mode = mode;
  return EVCONV_OK;
}

int32_t evconv_current_mode(const evconv_net* net) {
  if (!net) return -1;
  if (net->mode != EVCONV_MODE_AUTO) return net->mode;
  if (net->has_sparsify) return EVCONV_MODE_INCREMENTAL;
  return net->auto_phase == 0 ? EVCONV_MODE_INCREMENTAL : net->auto_phase == 1 ? EVCONV_MODE_DENSE_RECOMPUTE : net->auto_choice;
}

evconv_status evconv_set_refresh_period(evconv_net* net, int32_t period) {
  if (!net) return EVCONV_ERR_INVALID_ARG;
  if (period < 0) { net->err = "refresh period must be >= 0"; return EVCONV_ERR_INVALID_ARG; }
  net->refresh_period = period;
  net->since_refresh = 0;
  return EVCONV_OK;
}

evconv_status evconv_node_shape(const evconv_net* net, int32_t node, int32_t* chw) {
  if (!net || !chw || node < -1 || node >= (int)net->L.nodes.size()) return EVCONV_ERR_INVALID_ARG;
  const Geo& g = node < 0 ? net->L.gin : net->L.nodes[node].go;
  chw[0] = g.c; chw[1] = g.h; chw[2] = g.w;
  return EVCONV_OK;
}

evconv_status evconv_get_state(evconv_net* net, int32_t node, int32_t kind, void* dst, size_t bytes) {
  return evconv_get_state_stream(net, 0, node, kind, dst, bytes);
}

evconv_status evconv_stream_stride(const evconv_net* net, size_t* bytes, int32_t* n_streams) {
  if (!net || !bytes) return EVCONV_ERR_INVALID_ARG;
  *bytes = net->L.stride;
  if (n_streams) *n_streams = net->L.n_streams;
  return EVCONV_OK;
}

evconv_status evconv_get_state_stream(evconv_net* net, int32_t stream, int32_t node, int32_t kind, void* dst,
                                      size_t bytes) {
  if (!net) return EVCONV_ERR_INVALID_ARG;
  if (stream < 0 || stream >= net->L.n_streams) { net->err = "no such stream"; return EVCONV_ERR_INVALID_ARG; }
  if (!dst || node < -1 || node >= (int)net->L.nodes.size()) { net->err = "bad node or null dst"; return EVCONV_ERR_INVALID_ARG; }
  if (node >= 0 && net->L.nodes[node].gather_fused_into >= 0) {
    net->err = "this node is computed inside its consumer and keeps no state";
    return EVCONV_ERR_INVALID_ARG;
  }
  const Geo& g = node < 0 ? net->L.gin : net->L.nodes[node].go;
  const NodePlan* n = node < 0 ? nullptr : &net->L.nodes[node];
  const void* src = nullptr;
  size_t need = 0;
  const size_t elems = (size_t)g.c * g.sites();
  switch (kind) {
    case EVCONV_STATE_Z: src = n ? n->z : nullptr; need = elems * 4; break;
    case EVCONV_STATE_DY: src = n ? (const void*)n->out : (const void*)net->dx; need = elems * 4; break;
    case EVCONV_STATE_IDX: src = n ? n->idx : net->idx_in; need = (size_t)g.sites() * 4; break;
    case EVCONV_STATE_COUNT: src = n ? n->count : net->count_in; need = 4; break;
    case EVCONV_STATE_BITMAP: src = n ? n->bitmap : net->bitmap_in; need = ((size_t)g.tiles() + 63) / 64 * 8; break;
    case EVCONV_STATE_OCC: src = n ? n->occ : net->occ_in; need = (size_t)g.tiles() * 8; break;
    case EVCONV_STATE_OCC_TOUCHED: src = n ? n->touched : net->occ_in; need = (size_t)g.tiles() * 8; break;
    case EVCONV_STATE_X_PREV: src = n ? nullptr : net->x_prev; need = elems * 4; break;
    case EVCONV_STATE_STEP: src = n ? n->step : nullptr; need = 4; break;
    case EVCONV_STATE_Z2: src = n ? n->z2 : nullptr; need = elems * 4; break;
    default: net->err = "bad state kind"; return EVCONV_ERR_INVALID_ARG;
  }
  if (!src) { net->err = "this node keeps no such state"; return EVCONV_ERR_INVALID_ARG; }
  if (bytes != need) { net->err = "size mismatch: expected " + std::to_string(need) + " bytes"; return EVCONV_ERR_INVALID_ARG; }
  hipError_t e = hipStreamSynchronize(net->stream);
  if (e == hipSuccess)
    e = hipMemcpy(dst, (const char*)src + (size_t)stream * net->L.stride, need, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(net, e, "get_state");
  return EVCONV_OK;
}

evconv_status evconv_get_stats(evconv_net* net, int32_t node, evconv_layer_stats* out) {
  if (!net || !out || node < 0 || node >= (int)net->L.nodes.size()) return EVCONV_ERR_INVALID_ARG;
  const NodePlan& n = net->L.nodes[node];
  const int tiles = n.go.tiles();
  std::vector<uint64_t> words(2 * (size_t)tiles);
  hipError_t e = hipStreamSynchronize(net->stream);
  if (e == hipSuccess) e = hipMemcpy(words.data(), n.occ, words.size() * 8, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(net, e, "get_stats");
  memset(out, 0, sizeof *out);
  out->n_sites = n.go.sites();
  out->n_tiles = tiles;
  for (int t = 0; t < tiles; ++t) {
    out->n_active += __builtin_popcountll(words[t]);
    out->n_touched += __builtin_popcountll(words[tiles + t]);
    out->n_touched_tiles += words[tiles + t] != 0;
  }
  if (n.d.op == EVCONV_OP_CONV2D || n.d.op == EVCONV_OP_LINEAR) {
    const double per_site = 2.0 * n.d.kh * n.d.kh * n.d.c_in * n.d.c_out;
    out->flops_dense = per_site * n.go.sites();
    out->flops_executed = per_site * 64.0 * out->n_touched_tiles;
  }
  return EVCONV_OK;
}

evconv_status evconv_profile_begin(evconv_net* net, int32_t max_records) {
  if (!net || max_records <= 0) return EVCONV_ERR_INVALID_ARG;
  for (hipEvent_t e : net->prof_ev) (void)hipEventDestroy(e);
  net->prof_ev.assign(2 * (size_t)max_records, nullptr);
  for (hipEvent_t& e : net->prof_ev) {
    hipError_t err = hipEventCreate(&e);
    if (err != hipSuccess) return hip_fail(net, err, "hipEventCreate");
  }
  net->prof_node.clear();
  net->node_ms.assign(net->L.nodes.size() + 2, 0.0);  // [node + 1]
  net->node_launches.assign(net->L.nodes.size() + 2, 0);
  net->prof = true;
  return EVCONV_OK;
}

evconv_status evconv_profile_end(evconv_net* net) {
  if (!net) return EVCONV_ERR_INVALID_ARG;
  if (!net->prof) { net->err = "profiling was not started"; return EVCONV_ERR_STATE; }
  net->prof = false;
  hipError_t e = hipStreamSynchronize(net->stream);
  if (e != hipSuccess) return hip_fail(net, e, "profile_end");
  for (size_t r = 0; r < net->prof_node.size(); ++r) {
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, net->prof_ev[2 * r], net->prof_ev[2 * r + 1]);
    if (e != hipSuccess) return hip_fail(net, e, "hipEventElapsedTime");
    net->node_ms[net->prof_node[r] + 1] += ms;
    net->node_launches[net->prof_node[r] + 1] += 1;
  }
  for (hipEvent_t ev : net->prof_ev) (void)hipEventDestroy(ev);
  net->prof_ev.clear();
  net->prof_node.clear();
  return EVCONV_OK;
}

evconv_status evconv_get_node_time(const evconv_net* net, int32_t node, double* ms_total, int64_t* launches) {
  if (!net || !ms_total || !launches || node < -1 || node > (int)net->L.nodes.size()) return EVCONV_ERR_INVALID_ARG;
  if (net->node_ms.empty()) { *ms_total = 0; *launches = 0; return EVCONV_OK; }
  *ms_total = net->node_ms[node + 1];
  *launches = net->node_launches[node + 1];
  return EVCONV_OK;
}

const char* evconv_node_kernel(const evconv_net* net, int32_t node) {
  if (!net || node < 0 || node >= (int)net->L.nodes.size()) return "";
  if (net->L.nodes[node].fused_into >= 0) return "fused_into_conv_epilogue";
  if (net->L.nodes[node].gather_fused_into >= 0) {
    const NodePlan& consumer = net->L.nodes[net->L.nodes[node].gather_fused_into];
    if (consumer.d.op == EVCONV_OP_CONCAT) return "fused_into_concat_gather";
    // (folded into the conv's weights away from the image border, into its gather along the border)
    return consumer.fold_list ? "fused_into_conv_weights" : "fused_into_conv_gather";
  }
  return kKernelNames[net->L.nodes[node].kernel];
}

evconv_status evconv_debug_phase_stamps(int32_t operand_mode, uint64_t* out, int32_t max_records, int32_t reset,
                                        int32_t* n_records) {
  if (!n_records || max_records < 0 || (max_records > 0 && !out)) return EVCONV_ERR_INVALID_ARG;
  int n;
  unsigned long long* dst = (unsigned long long*)out;
  if (operand_mode == EVCONV_F32) n = evk::conv_mfma_f32_phase_stamps(dst, max_records, reset != 0);
  else if (operand_mode == EVCONV_BF16) n = evk::conv_mfma_bf16_phase_stamps(dst, max_records, reset != 0);
  else if (operand_mode == EVCONV_F32_SPLIT) n = evk::conv_mfma_split_phase_stamps(dst, max_records, reset != 0);
  else return EVCONV_ERR_INVALID_ARG;
  if (n == -1) return EVCONV_ERR_UNSUPPORTED;
  if (n < 0) return EVCONV_ERR_HIP;
  *n_records = n;
  return EVCONV_OK;
}

evconv_status evconv_debug_chip_probes(void* scratch, size_t scratch_bytes, void* hip_stream, float* out, int32_t n_out) {
  if (!scratch || !out || scratch_bytes < EVCONV_CHIP_PROBE_SCRATCH_BYTES || n_out < EVCONV_CHIP_PROBE_VALUES)
    return EVCONV_ERR_INVALID_ARG;
  static_assert(EVCONV_CHIP_PROBE_VALUES == evk::kChipProbeValues && EVCONV_CHIP_PROBE_SCRATCH_BYTES == evk::kChipProbeScratch,
                "header and probes disagree");
  return evk::chip_probes(scratch, scratch_bytes, (hipStream_t)hip_stream, out, n_out) == evk::kChipProbeValues ? EVCONV_OK
                                                                                                                 : EVCONV_ERR_HIP;
}

const char* evconv_last_error(const evconv_net* net) { return net ? net->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
