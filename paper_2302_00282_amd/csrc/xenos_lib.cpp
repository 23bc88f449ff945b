// Host side of the library: graph ingest, the automatic optimiser (fusion pre-pass, operator
// linking, DSP-aware operator split; Sections 4.1-4.4 of the paper) and the runtime that enqueues
// the planned kernel sequence (Section 3).  Pure C++ plus the HIP runtime API; all arithmetic on
// tensor data happens in the gfx950 kernels.
#include <hip/hip_runtime.h>
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/xenos.h"
#include "kernels.h"

using namespace xenos;

namespace {

thread_local std::string g_err;

xenos_status fail(xenos_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return st;
}

constexpr uint32_t MAGIC_GRAPH = 0x58474631u, MAGIC_PLAN = 0x58504c31u;

struct Shape { int n = 0, c = 0, h = 0, w = 0; };

struct GOp {
  xenos_op_desc d;
  std::vector<float> weight, bias, gamma, beta, mean, var;
};

int pool_out(int n, int k, int s, int p, int ceil_mode) {
  if (ceil_mode) {
    int o = (n + 2 * p - k + s - 1) / s + 1;
    if ((o - 1) * s >= n + p) --o;
    return o;
  }
  return (n + 2 * p - k) / s + 1;
}

}  // namespace

struct xenos_graph {
  uint32_t magic = MAGIC_GRAPH;
  xenos_tensor_desc in{}, out{};
  std::vector<GOp> ops;
  std::vector<Shape> shapes;   // by tensor id
  int output_id = 0;
};

// ---------------------------------------------------------------------------------------------
// Plan structures
// ---------------------------------------------------------------------------------------------
namespace {

enum StepKind { S_CONV = 0, S_DW = 1, S_ELT = 2, S_POOL = 3, S_CVT = 4, S_SPLITK = 5 };
const char* kStepNames[] = {"conv", "dwconv", "elt", "pool", "cvt", "splitk_finish"};
const char* kModeNames[] = {"flat", "zigzag", "patch", "gap"};

struct Buffer {
  long long bytes = 0;
  int ext = 0;                 // 0 workspace, 1 graph input, 2 graph output
  size_t offset = 0;
  int first = 1 << 30, last = -1;
};

// A logical tensor as laid out in memory: element strides for image, pixel (h*W+w) and channel.
struct View {
  int buf = -1;
  long long off = 0;           // element offset into the buffer (channel offset of a concat slice)
  long long sN = 0, sP = 0, sK = 1;
  int f32 = 0;                 // elements are fp32 (only possible for graph input / output)
  int esz = 4;
  Shape s;
  int cphys = 0;               // channels physically present per pixel (> s.c: zero-filled padding channels follow)
  // which tensor of the caller's graph the view holds (plan metadata, for per-chain checks): channel c of the view is
  // channel gc0 + c * gcs of graph tensor gt; gt < 0 = no graph tensor (partial sums of a reduction split)
  int gt = -1, gc0 = 0, gcs = 1;
  bool internal_nhwc() const { return sK == 1; }
};

struct Step {
  int kind = S_CONV;
  std::string name;
  std::vector<int> ops;        // graph operator ids executed by this step
  ConvArgs conv{};
  DwArgs dw{};
  EltArgs elt{};
  PoolArgs pool{};
  CvtArgs cvt{};
  SplitKArgs splitk{};
  int cfg = 0, scalar = 0, stem = 0;
  int stem_lds = 0;            // first-layer chain on the kernel that stages its input block in LDS
  int fc_stream = 0;           // fully connected chain with few rows: weights streamed by fc_stream_kernel, finished by the summing pass
  int gap_finish = 0;          // global average linked through the summing pass of a reduction split (few images)
  // every partition the split planner found legal for this chain (tile shape x kernel), for profiling-driven choice;
  // empty when the choice is forced or tied to the structure of the plan (reduction split, stem, linked depthwise)
  struct Cand { int cfg; ConvArgs a; size_t lds; };
  std::vector<Cand> cands;
  int tuned = 0;               // chosen by measurement (xenos_plan_tune)
  int v_in = -1, v_in2 = -1, v_out = -1;
  int v_out2 = -1;             // second output of a Fire-module chain (the 3x3 expand's part)
  long long w_off = -1, scale_off = -1, shift_off = -1, ktab_off = -1;   // byte offsets into the weight image
  long long fire_w_off[2] = {-1, -1}, fire_scale_off[2] = {-1, -1}, fire_shift_off[2] = {-1, -1};   // expand chains of a Fire module
  long long dw_w_off = -1, dw_scale_off = -1, dw_shift_off = -1;        // linked depthwise producer, if any
  double flops = 0;
  long long bytes_in = 0, bytes_w = 0, bytes_out = 0, bytes_res = 0;
  size_t lds = 0;
};

// Internal node list (a rewritten copy of the graph: pooling hoisted above concat when linking).
struct Node {
  int kind = 0;
  std::vector<int> in;
  int src = -1;                // graph op that supplies attributes / parameters
  Shape out;
};

}  // namespace

struct xenos_plan {
  uint32_t magic = MAGIC_PLAN;
  xenos_plan_opts opts{};
  xenos_hw_info hw{};
  xenos_tensor_desc in{}, out{};
  int dt = DT_F32, esz = 4, ce = 4;
  int n_linked_shuffles = 0;   // channel shuffles realised as the store order of their concat (no pass of their own)
  size_t zero_off = 0;         // 256 zero bytes at the start of the weight image
  std::vector<Buffer> bufs;
  std::vector<View> views;
  std::vector<Step> steps;
  std::vector<unsigned char> wimage;   // exact image of the device weight buffer
  size_t workspace_bytes = 0;
  std::string json;
  void* d_weights = nullptr;
  void* d_workspace = nullptr;
  bool bound = false;
  // xenos_run_graph: one instantiated HIP graph per (input, output) pointer pair, captured on a private stream
  std::map<std::pair<const void*, void*>, hipGraphExec_t> graphs;
  hipStream_t capture_stream = nullptr;
  ~xenos_plan() {
    for (auto& kv : graphs) (void)hipGraphExecDestroy(kv.second);
    if (capture_stream) (void)hipStreamDestroy(capture_stream);
  }
};

namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

uint16_t f2bf_host(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

void write_plan_json(xenos_plan& p);

// ---------------------------------------------------------------------------------------------
// Planner
// ---------------------------------------------------------------------------------------------
struct Planner {
  const xenos_graph& g;
  xenos_plan& p;
  std::vector<Node> nodes;
  std::vector<Shape> tshape;                 // by tensor id (node list numbering)
  struct GraphRef { int gt, c0; };
  std::vector<GraphRef> tgraph;              // by tensor id: the graph tensor (and first channel of it) the tensor is
  std::vector<std::vector<int>> consumers;   // tensor id -> node indices
  int out_tid = 0;
  std::vector<int> tview;                    // tensor id -> view index (-1 = not materialised)
  std::vector<int> node_step;                // node -> step index (-1 = not yet planned)
  std::vector<int> node_final;               // node -> 1 if its output is its step's output
  struct Place { int cat_tid; int c_off; int c_stride; };
  std::map<int, Place> placed;               // tensor id -> slice of a concat output (channel c of it at c_off + c * c_stride)
  std::vector<char> free_concat;             // node -> concat realised by offset writes
  std::vector<int> ileave;                   // concat node -> groups of the channel shuffle linked into it (0 = none):
                                             // part j of the concat is written to channels j, j + groups, j + 2 groups, ...
  std::vector<char> alias_shuffle;           // shuffle node whose output IS its (already interleaved) concat input
  // Two-group shuffle finished by one chain: the chain that ends in tensor `key` stores its channels AND those of the
  // other part (tensor `other`, complete before the chain runs) alternately into the concat buffer `cat_tid`
  struct Fin { int cat_tid; int pos; int other; };
  std::map<int, Fin> fin;
  std::vector<char> fin_concat;              // concat node whose two parts are written by such a chain
  std::vector<char> fold_shuffle;            // shuffle node folded into the weights of the dense convolutions that read it
  int pack_shuffle_groups = 0;               // pack_dense: the input channels are read through a shuffle of this many groups

  Planner(const xenos_graph& g_, xenos_plan& p_) : g(g_), p(p_) {}

  const xenos_op_desc& desc(const Node& n) const { return g.ops[n.src].d; }

  size_t wpush(const void* data, size_t bytes) {
    size_t off = align_up(p.wimage.size(), 256);
    p.wimage.resize(off + bytes);
    if (data) memcpy(p.wimage.data() + off, data, bytes);
    return off;
  }

  // ---- node list -----------------------------------------------------------------------------
  void build_nodes() {
    const int n_ops = (int)g.ops.size();
    std::vector<std::vector<int>> cons(n_ops + 1);
    for (int i = 0; i < n_ops; ++i)
      for (int j = 0; j < g.ops[i].d.n_inputs; ++j) cons[g.ops[i].d.inputs[j]].push_back(i);
    auto is_pool = [&](int k) { return k == XENOS_OP_MAXPOOL || k == XENOS_OP_AVGPOOL || k == XENOS_OP_GLOBAL_AVGPOOL; };
    // concat -> pool hoisting (pooling is per channel, so it commutes with a channel concat); lets the
    // pooling link into each producer of the concat
    std::vector<int> hoist_pool(n_ops, -1);   // concat op -> pool op
    std::vector<char> skip(n_ops, 0);
    if (p.opts.link >= 2)
      for (int i = 0; i < n_ops; ++i) {
        if (g.ops[i].d.kind != XENOS_OP_CONCAT || g.output_id == i + 1) continue;
        if (cons[i + 1].size() == 1 && is_pool(g.ops[cons[i + 1][0]].d.kind)) {
          hoist_pool[i] = cons[i + 1][0];
          skip[cons[i + 1][0]] = 1;
        }
      }
    std::vector<int> remap(n_ops + 1, -1);
    remap[0] = 0;
    tshape.clear();
    tshape.push_back(g.shapes[0]);
    tgraph.clear();
    tgraph.push_back(GraphRef{0, 0});
    auto push = [&](Node nd, int gt, int c0) {
      nodes.push_back(nd);
      tshape.push_back(nd.out);
      tgraph.push_back(GraphRef{gt, c0});
      return (int)nodes.size();
    };
    for (int i = 0; i < n_ops; ++i) {
      if (skip[i]) continue;   // remap set when its concat was emitted
      const xenos_op_desc& d = g.ops[i].d;
      if (hoist_pool[i] >= 0) {
        const int po = hoist_pool[i];
        Node cat;
        cat.kind = XENOS_OP_CONCAT; cat.src = i; cat.out = g.shapes[po + 1];
        int c0 = 0;
        for (int j = 0; j < d.n_inputs; ++j) {
          Node pl;
          pl.kind = g.ops[po].d.kind; pl.src = po;
          pl.in = {remap[d.inputs[j]]};
          pl.out = g.shapes[po + 1];
          pl.out.c = g.shapes[d.inputs[j]].c;
          cat.in.push_back(push(pl, po + 1, c0));   // the pooled part = a channel range of the pooled concat
          c0 += pl.out.c;
        }
        const int t = push(cat, po + 1, 0);
        remap[i + 1] = t;
        remap[po + 1] = t;
        continue;
      }
      Node nd;
      nd.kind = d.kind; nd.src = i; nd.out = g.shapes[i + 1];
      for (int j = 0; j < d.n_inputs; ++j) nd.in.push_back(remap[d.inputs[j]]);
      remap[i + 1] = push(nd, i + 1, 0);
    }
    out_tid = remap[g.output_id];
    consumers.assign(nodes.size() + 1, {});
    for (int i = 0; i < (int)nodes.size(); ++i)
      for (int t : nodes[i].in) consumers[t].push_back(i);
  }

  // ---- views / buffers -----------------------------------------------------------------------
  int new_buffer(long long bytes, int ext) {
    Buffer b;
    b.bytes = bytes; b.ext = ext;
    p.bufs.push_back(b);
    return (int)p.bufs.size() - 1;
  }

  int ext_view(const xenos_tensor_desc& d, int ext) {
    View v;
    v.s = Shape{d.n, d.c, d.h, d.w};
    v.f32 = d.dtype == XENOS_F32 ? 1 : 0;
    v.esz = d.dtype == XENOS_F32 ? 4 : 2;
    if (d.layout == XENOS_NHWC) { v.sK = 1; v.sP = d.c; v.sN = (long long)d.h * d.w * d.c; }
    else { v.sK = (long long)d.h * d.w; v.sP = 1; v.sN = (long long)d.c * d.h * d.w; }
    v.buf = new_buffer((long long)d.n * d.c * d.h * d.w * v.esz, ext);
    p.views.push_back(v);
    return (int)p.views.size() - 1;
  }
  // is the external tensor directly usable as an internal NHWC tensor of the compute type?
  bool ext_is_internal(const xenos_tensor_desc& d) const {
    const bool dt_ok = (d.dtype == XENOS_F32 && p.dt == DT_F32) || (d.dtype == XENOS_BF16 && p.dt == DT_BF16);
    const bool lay_ok = d.layout == XENOS_NHWC || (d.h == 1 && d.w == 1);
    return dt_ok && lay_ok;
  }
  int internal_view(const Shape& s, int buf = -1, int ctot = 0, int c_off = 0) {
    View v;
    v.s = s; v.esz = p.esz; v.f32 = 0;
    if (ctot == 0) ctot = s.c;
    v.sK = 1; v.sP = ctot; v.sN = (long long)s.h * s.w * ctot; v.off = c_off;
    v.buf = buf >= 0 ? buf : new_buffer((long long)s.n * s.h * s.w * ctot * p.esz, 0);
    p.views.push_back(v);
    return (int)p.views.size() - 1;
  }
  // Fix up an external view so that steps treating it as "internal" see NHWC strides (1x1 maps in NCHW).
  void normalise_1x1(View& v) {
    if (v.s.h == 1 && v.s.w == 1) { v.sK = 1; v.sP = v.s.c; v.sN = v.s.c; }
  }

  // records which graph tensor view `v` holds: tensor `tid` of the node list, from its channel `c_first` on
  int tag(int v, int tid, int c_first = 0, int c_stride = 1) {
    p.views[v].gt = tgraph[tid].gt; p.views[v].gc0 = tgraph[tid].c0 + c_first; p.views[v].gcs = c_stride;
    return v;
  }

  // View a step should write tensor `tid` to.  Creates it on first request.
  int out_view_for(int tid, bool producer_is_conv) {
    if (tview[tid] >= 0) return tview[tid];
    const Shape s = tshape[tid];
    int v;
    auto it = placed.find(tid);
    auto fi = fin.find(tid);
    if (fi != fin.end()) {
      v = out_view_for(fi->second.cat_tid, false);               // the chain writes the whole concat buffer
    } else if (it != placed.end()) {
      const int cat = it->second.cat_tid;
      const int cv = out_view_for(cat, false);
      const View& c = p.views[cv];
      View sl = c;
      sl.s = s; sl.off = c.off + it->second.c_off * c.sK; sl.sK = c.sK * it->second.c_stride;
      p.views.push_back(sl);
      v = (int)p.views.size() - 1;
    } else if (tid == out_tid) {
      if (producer_is_conv || ext_is_internal(p.out)) {
        v = ext_view(p.out, 2);
        if (ext_is_internal(p.out)) { normalise_1x1(p.views[v]); p.views[v].f32 = 0; }
      } else {
        v = internal_view(s);
        need_export = true;
      }
    } else {
      v = internal_view(s);
    }
    if (fi == fin.end()) {
      tag(v, tid);
      // a concat written interleaved holds the output of the channel shuffle linked into it
      if (tid >= 1 && nodes[tid - 1].kind == XENOS_OP_CONCAT && ileave[tid - 1] && consumers[tid].size() == 1) tag(v, consumers[tid][0] + 1);
    }
    tview[tid] = v;
    return v;
  }
  bool need_export = false;

  // A depthwise chain waiting to be linked into the pointwise convolution that consumes it (link level 3)
  bool in_lazy = false, in_all_dense = false, in_gather = false;   // graph input not yet imported; see plan()

  struct DwPro {
    bool active = false;
    int v_in = -1;
    std::vector<int> ops;
    long long w_off = -1, scale_off = -1, shift_off = -1;
    int k = 0, stride = 0, pad = 0, H = 0, W = 0, relu = 0;
    double flops = 0;
    long long bytes_w = 0;
  } dwpro;

  // A first-layer 3x3 chain waiting to be linked into the 3x3 convolution that consumes it (link level 3; Table 1,
  // ConvX -> ConvY): its output tensor is then never materialised
  struct PairPro {
    bool active = false;
    std::vector<int> ops;
    long long w_off = -1, scale_off = -1, shift_off = -1;
    int relu = 0;
    double flops = 0;
    long long bytes_w = 0;
  } pairpro;

  // Can the dense convolution node `nx` take a linked first-layer producer?  It must be a 3x3 / stride 1 / pad 1
  // convolution kPairChannels -> kPairChannels whose own chain ends in nothing or a 2x2 / stride 2 pooling of an even map,
  // takes no shortcut, and writes a plain internal tensor (the walk mirrors the link pass of plan_node).
  // Can the chain that produces tensor `tid` store it with a channel stride?  True for conv -> (bias | bn)* -> [relu]
  // on a dense convolution that does not read the graph input (the general convolution kernel stores single elements
  // at any stride; the first-layer, halo, depthwise and pooling epilogues store 16-byte channel groups only), when
  // nothing else reads the tensor or the intermediate ones.
  bool stores_strided(int tid) const { return plain_chain_conv(tid) >= 0; }
  // (the convolution node of that chain, or -1)
  int plain_chain_conv(int tid) const {
    if (tid < 1 || tid == out_tid || placed.count(tid) || consumers[tid].size() != 1) return -1;
    int t = tid;
    if (nodes[t - 1].kind == XENOS_OP_RELU) {
      t = nodes[t - 1].in[0];
      if (t < 1 || t == out_tid || consumers[t].size() != 1) return -1;
    }
    while (nodes[t - 1].kind == XENOS_OP_BIAS || nodes[t - 1].kind == XENOS_OP_BN) {
      t = nodes[t - 1].in[0];
      if (t < 1 || t == out_tid || consumers[t].size() != 1) return -1;
    }
    const Node& c = nodes[t - 1];
    return c.kind == XENOS_OP_CONV && desc(c).groups == 1 && c.in[0] != 0 ? t - 1 : -1;
  }

  // Does the chain that starts at convolution node `c` end in a tensor stored with a channel stride?
  bool chain_stores_strided(int c) const {
    int cur = c + 1;
    for (;;) {
      auto it = placed.find(cur);
      if (it != placed.end()) return it->second.c_stride > 1;
      const int nx = single_consumer(cur);
      if (nx < 0) return false;
      const int k = nodes[nx].kind;
      if (k != XENOS_OP_BIAS && k != XENOS_OP_BN && k != XENOS_OP_RELU) return false;
      cur = nx + 1;
    }
  }

  // Does the chain that starts at convolution node `c` link a window pooling (max / average with a window, not the
  // global average)?  Mirrors the link pass of plan_node.
  bool chain_links_window_pool(int c) const {
    int cur = c + 1, stage = 0;
    for (;;) {
      if (cur == out_tid || placed.count(cur)) return false;
      const int nx = single_consumer(cur);
      if (nx < 0) return false;
      const int k = nodes[nx].kind;
      if ((k == XENOS_OP_BIAS || k == XENOS_OP_BN) && stage == 0) {
      } else if (k == XENOS_OP_ADD && stage <= 1) { stage = 2;
      } else if (k == XENOS_OP_RELU && stage <= 2) { stage = 3;
      } else if ((k == XENOS_OP_MAXPOOL || k == XENOS_OP_AVGPOOL) && stage <= 3) { return true;
      } else return false;
      cur = nx + 1;
    }
  }

  bool pair_consumer_ok(int nx) {
    const Node& nd = nodes[nx];
    if (nd.kind != XENOS_OP_CONV || node_step[nx] >= 0) return false;
    const xenos_op_desc& d = desc(nd);
    const Shape is = tshape[nd.in[0]];
    if (d.groups != 1 || d.kh != 3 || d.kw != 3 || d.stride_h != 1 || d.stride_w != 1 || d.pad_h != 1 || d.pad_w != 1 ||
        d.out_c != kPairChannels || is.c != kPairChannels || is.h < 4) return false;
    int cur = nx + 1, stage = 0;
    for (;;) {
      if (cur == out_tid || placed.count(cur)) return false;
      const int c = single_consumer(cur);
      if (c < 0) return true;
      const Node& nn_ = nodes[c];
      if ((nn_.kind == XENOS_OP_BIAS || nn_.kind == XENOS_OP_BN) && stage == 0) {
      } else if (nn_.kind == XENOS_OP_ADD && stage <= 1) {
        return false;
      } else if (nn_.kind == XENOS_OP_RELU && stage <= 2) {
        stage = 3;
      } else if (nn_.kind == XENOS_OP_GLOBAL_AVGPOOL && stage <= 3) {
        return false;
      } else if ((nn_.kind == XENOS_OP_MAXPOOL || nn_.kind == XENOS_OP_AVGPOOL) && stage <= 3) {
        const xenos_op_desc& pd = desc(nn_);
        const Shape ps = tshape[c + 1];
        if (pd.kh != 2 || pd.kw != 2 || pd.stride_h != 2 || pd.stride_w != 2 || pd.pad_h != 0 || pd.pad_w != 0 || is.h % 2 || is.w % 2 ||
            2 * ps.h != is.h || 2 * ps.w != is.w) return false;
        return c + 1 != out_tid && !placed.count(c + 1);
      } else {
        return true;
      }
      cur = c + 1;
    }
  }

  void touch(int view, int step) {
    Buffer& b = p.bufs[p.views[view].buf];
    b.first = std::min(b.first, step);
    b.last = std::max(b.last, step);
  }

  long long view_bytes(int v) const {
    const View& vw = p.views[v];
    return (long long)vw.s.n * vw.s.c * vw.s.h * vw.s.w * vw.esz;
  }

  // ---- the fusion pre-pass: fold Bias / Bn into one per-channel scale and shift (fp64) --------
  struct Affine { std::vector<double> scale, shift; };
  static void fold_bias(Affine& a, const std::vector<float>& b) {
    for (size_t k = 0; k < a.shift.size(); ++k) a.shift[k] += (double)b[k];
  }
  static void fold_bn(Affine& a, const GOp& o) {
    for (size_t k = 0; k < a.shift.size(); ++k) {
      const double s = (double)o.gamma[k] / sqrt((double)o.var[k] + (double)o.d.eps);
      a.scale[k] *= s;
      a.shift[k] = (a.shift[k] - (double)o.mean[k]) * s + (double)o.beta[k];
    }
  }
  void push_affine(const Affine& a, int padded, long long* scale_off, long long* shift_off) {
    std::vector<float> sc(padded, 1.f), sh(padded, 0.f);
    for (size_t k = 0; k < a.scale.size(); ++k) { sc[k] = (float)a.scale[k]; sh[k] = (float)a.shift[k]; }
    *scale_off = (long long)wpush(sc.data(), sc.size() * 4);
    *shift_off = (long long)wpush(sh.data(), sh.size() * 4);
  }

  // ---- operator split for one dense-conv chain ------------------------------------------------
  bool choose_patch(int bm, int pk, int ps, int PH, int PW, int* pph, int* ppw) {
    int best = 0;
    for (int a = 1; a <= PH; ++a)
      for (int b = 1; b <= PW; ++b) {
        const int hh = (a - 1) * ps + pk, ww = (b - 1) * ps + pk;
        if (hh * ww > bm) continue;
        const int score = a * b * 64 - abs(a - b);
        if (score > best) { best = score; *pph = a; *ppw = b; }
      }
    return best > 0;
  }

  // Workgroup slots of a conv launch.  The dense-conv kernel deals its workgroups to an xcd_m x (8/xcd_m) grid of
  // XCDs over pixel tiles x (channel tiles x reduction shares); pick the factorisation with the shortest longest
  // queue, preferring the pixel split (workgroups of one XCD then share a weight slice).
  void set_grid(ConvArgs& c, int cfg) {
    const int ks = c.ksplit > 1 ? c.ksplit : 1;
    if (cfg == kHaloCfg) {
      // persistent workgroups, one per compute unit, an equal number on every XCD
      c.xcd_m = 8;
      const int per_xcd = std::max(1, std::min(std::max(1, p.hw.num_cu) / 8, (c.tiles_m + 7) / 8 * c.tiles_n * ks));
      c.grid = 8 * per_xcd;
      // Order of an XCD's tiles.  One sweep of its pixel tiles per output-channel tile keeps a single weight slice
      // live in the XCD's L2 (4 MB), and re-reads the input once per channel tile when the XCD's share of the input
      // is larger than that.  When all the weights take at most half the L2, the workgroups of one round cover every
      // channel tile of a group of pixel tiles instead, and each input patch is fetched once (measured with the L2
      // fetch counter on 56x56 maps of 256 channels: 2.5 -> 1.2-1.7 times the input; layers with larger weights
      // fetch the same or a little more that way, and run times do not differ).
      const long long w_bytes = (long long)c.K * c.C * 9 * p.esz;
      const long long l2 = p.hw.l2_bytes ? (long long)p.hw.l2_bytes : kL2BytesPerXcd;
      c.halo_mgroup = c.tiles_n >= 2 && w_bytes <= l2 / 2 ? std::max(1, per_xcd / c.tiles_n) : 1 << 30;
    } else {
      const int nz = c.tiles_n * ks;
      long long best = -1;
      for (int xm = 8; xm >= 1; xm /= 2) {
        const int xn = 8 / xm;
        const long long q = (long long)((c.tiles_m + xm - 1) / xm) * ((nz + xn - 1) / xn);
        if (best < 0 || q < best) { best = q; c.xcd_m = xm; }
      }
      c.grid = (int)(best * 8);
    }
    if (!p.opts.split) c.grid = 1;
  }

  // What the halo-staged 3x3 kernel needs of a chain's input side (its output side depends on who stores the result)
  bool halo_input_ok(const Step& st) const {
    const ConvArgs& c = st.conv;
    return !c.ileave && !c.dw_w && !c.pair && c.R == 3 && c.S == 3 && c.stride == 1 && c.pad == 1 && !st.scalar && c.C % (kRowBytes / p.esz) == 0 &&
           (long long)c.N * c.in_sN < (1ll << 31) && conv_lds_bytes(kHaloCfg, M_FLAT) <= p.hw.lds_bytes_per_cu;
  }
  // Tile of the plain form of the halo kernel for a pixel-major (step 1) or zig-zag (step 2) chain: the TH x TW block of
  // at most kHaloRows pixels that wastes the fewest GEMM rows over the images stacked with their padding rows
  bool choose_halo_tile(const ConvArgs& c, int step, ConvArgs& t) const {
    const long long rows = (long long)c.N * (c.H + 2);
    double best_fill = 0;
    for (int tw = step; tw <= std::min(c.W + step - 1, kHaloRows); tw += step) {
      if (tw + 2 > kHaloPitchWide) break;
      // (the staged patch has one of three row pitches; the smallest is for maps up to 8 wide, whose tiles are then more rows
      // high within the same patch: 34 x 7 pixels of a 7x7 map instead of 18 x 7.  Wider maps measured the same with 32 x 8
      // tiles at that pitch as with 16 x 16 tiles, and keep the squarer tile, which re-reads less halo)
      const int pitch = (c.W <= 8 && tw + 2 <= kHaloPitchTiny) ? kHaloPitchTiny : tw + 2 <= kHaloPitchNarrow ? kHaloPitchNarrow : kHaloPitchWide;
      int th = kHaloRows / tw / step * step;
      while (th >= step && (th + 2) * pitch > kHaloPatchMax) th -= step;
      if (th < step) continue;
      const long long ty = (rows + th - 1) / th, tx = (c.W + tw - 1) / tw;
      const double fill = (double)c.N * c.H * c.W / ((double)ty * tx * kHaloRows);
      if (fill > best_fill + 1e-9) { best_fill = fill; t.th = th; t.tw = tw; t.tiles_y = (int)ty; t.tiles_x = (int)tx; }
    }
    return best_fill > 0;
  }

  // Reduction split inside the halo kernel (Section 4.2.2: a split over C needs an extra reduction).  For maps so small
  // that the pixel x channel tiles of a 3x3 layer leave most units idle (7x7 x 512 at batch 32: 32 tiles of 128
  // channels), each tile's channel chunks are shared out over `ks` workgroups and a summing pass finishes the chain.
  // The choice is a time model in microseconds on the measured rates of the kernel: a 256 x 128 tile does one chunk of
  // 9 taps x 128 bytes of channels in 7.4 us (bf16; 4.6 us with 64 channels), a tile costs about 3 us around its chunks,
  // the summing pass one launch and the partial sums written and read back.  Returns ks (0 = do not split).
  struct HaloSplit { int ks = 0, bn = 0; ConvArgs tile{}; };
  HaloSplit choose_halo_split(const Step& st) const {
    HaloSplit r;
    const ConvArgs& c = st.conv;
    const int num_cu = std::max(1, p.hw.num_cu);
    if (!p.opts.split || p.opts.tile != 0 || !halo_input_ok(st) || c.OH != c.H || c.OW != c.W) return r;
    const int bke = kRowBytes / p.esz, nch = c.C / bke;
    if (nch < 2) return r;
    ConvArgs t = c;
    if (!choose_halo_tile(c, 1, t)) return r;
    t.tiles_m = t.tiles_y * t.tiles_x;
    t.halo_plin = 0;
    // (measured on ResNet-18: with fewer pixel tiles, batch 1 to 8 on 7x7 and 14x14 maps, the small gather tiles with
    // their own reduction split are faster than shares of 256-row tiles that are mostly dummy rows)
    if (t.tiles_m < 8) return r;
    const double chunk_flops = 2.0 * kHaloRows * 9 * bke;                      // per output channel of the tile
    const double rate[2] = {p.dt == DT_BF16 ? 5.1e6 : 0.45e6, p.dt == DT_BF16 ? 4.1e6 : 0.40e6};   // flop / us / unit
    static const int bns[2] = {128, 64};
    const double kTileUs = 3.0, kLaunchUs = 3.0, kPartBytesPerUs = 4.0e6;
    double best = 1e300, unsplit = 1e300;
    for (int v = 0; v < 2; ++v) {
      const int tn = (c.K + bns[v] - 1) / bns[v];
      const long long tiles = (long long)t.tiles_m * tn;
      const double chunk_us = chunk_flops * bns[v] / rate[v];
      for (int ks = 1; ks <= nch; ++ks) {
        if (nch % ks) continue;
        const long long rounds = (tiles * ks + num_cu - 1) / num_cu;
        double us = rounds * (kTileUs + nch / ks * chunk_us);
        if (ks == 1) { unsplit = std::min(unsplit, us); continue; }
        us += kLaunchUs + 2.0 * ks * c.N * c.OH * c.OW * (double)(tn * bns[v]) * 4 / kPartBytesPerUs;
        if (us < best) { best = us; r.ks = ks; r.bn = bns[v]; }
      }
    }
    // (the unsplit forms are also what the tuner picks among: give them the benefit of the doubt)
    if (r.ks < 2 || best > 0.8 * unsplit) { r.ks = 0; return r; }
    t.halo_bn = r.bn;
    t.tiles_n = (c.K + r.bn - 1) / r.bn;
    t.ntiles = t.tiles_m * t.tiles_n;
    r.tile = t;
    return r;
  }

  xenos_status split_conv(Step& st) {
    ConvArgs& c = st.conv;
    const int num_cu = std::max(1, p.hw.num_cu);
    if (st.stem && st.stem_lds) {   // tiles of 8 x 16 output pixels (3 x 8 pooling windows) of one image, persistent workgroups
      c.th = kStemLdsTh; c.tw = kStemLdsTw;
      c.tiles_y = (c.OH + c.th - 1) / c.th; c.tiles_x = (c.OW + c.tw - 1) / c.tw;
      if (c.pool != POOL_NONE) {
        c.pph = kStemLdsPph; c.ppw = kStemLdsPpw;
        c.tiles_y = (c.PH + c.pph - 1) / c.pph; c.tiles_x = (c.PW + c.ppw - 1) / c.ppw;
      }
      c.tiles_m = c.N * c.tiles_y * c.tiles_x; c.tiles_n = 1; c.ntiles = c.tiles_m; c.xcd_m = 8;
      c.grid = p.opts.split ? std::max(1, std::min(c.tiles_m, 4 * num_cu)) : 1;
      st.cfg = kStemLdsCfg;
      st.lds = conv_lds_bytes(kStemLdsCfg, c.mode);
      return XENOS_OK;
    }
    if (st.stem) {   // one wavefront = 32 pixels x all channels; workgroups of 4 wavefronts stride over the pixel blocks
      c.tiles_m = (c.M_total + 31) / 32; c.tiles_n = 1; c.ntiles = c.tiles_m; c.xcd_m = 8;
      c.grid = p.opts.split ? std::max(1, std::min((c.tiles_m + 3) / 4, 4 * num_cu)) : 1;   // 4 resident workgroups per unit
      st.cfg = kStemCfg;
      st.lds = conv_lds_bytes(kStemCfg, c.mode);
      return XENOS_OK;
    }
    if (c.pair) {
      // two linked 3x3 convolutions: a TH x TW block of output pixels (at most 128) x all 64 channels per workgroup, tiles
      // laid over the images stacked with their padding rows; the kernel stages a (TH+4) x (TW+4) block of the graph
      // input and a (TH+2) x 18 patch of the intermediate tensor, and keeps both weight tensors in registers
      if (!c.vec_out || c.has_res || (c.mode != M_FLAT && c.mode != M_ZIGZAG) || (c.mode == M_ZIGZAG && (c.H % 2 || c.W % 2)) ||
          conv_lds_bytes(kPairCfg, c.mode) > p.hw.lds_bytes_per_cu)
        return fail(XENOS_EUNSUPPORTED, "%s: chain cannot take a linked first-layer producer", st.name.c_str());
      const int step = c.mode == M_ZIGZAG ? 2 : 1;
      const long long rows = (long long)c.N * (c.H + 2);
      double best_fill = 0;
      for (int tw = step; tw + 2 <= kHaloPitchNarrow && tw < c.W + step; tw += step) {
        int th = std::min(kPairRows / tw, c.H - 2) / step * step;   // a tile's input rows lie in at most two images
        while (th >= step && ((th + 2) * kHaloPitchNarrow > kPairPatchMax || (th + 4) * (tw + 4) > kPairInMax || (th + 3) * (tw + 4) + 20 > kPairInMax)) th -= step;
        if (th < step) continue;
        const long long ty = (rows + th - 1) / th, tx = (c.W + tw - 1) / tw;
        const double fill = (double)c.N * c.H * c.W / ((double)ty * tx * kPairRows);
        if (fill > best_fill + 1e-9) { best_fill = fill; c.th = th; c.tw = tw; c.tiles_y = (int)ty; c.tiles_x = (int)tx; }
      }
      if (best_fill <= 0) return fail(XENOS_EUNSUPPORTED, "%s: no tile of the pair kernel fits", st.name.c_str());
      c.tiles_m = c.tiles_y * c.tiles_x; c.tiles_n = 1; c.ntiles = c.tiles_m; c.xcd_m = 8;
      c.grid = p.opts.split ? 8 * std::max(1, std::min(2 * num_cu / 8, (c.tiles_m + 7) / 8)) : 1;   // two workgroups per unit
      st.cfg = kPairCfg;
      st.lds = conv_lds_bytes(kPairCfg, c.mode);
      return XENOS_OK;
    }
    // halo-staged 3x3 kernel: a TH x TW block of output pixels (256 GEMM rows) x 128 channels per workgroup,
    // tiles laid over the images stacked with their padding rows
    // (the halo kernel stores 16-byte channel groups only: outputs and shortcuts that cannot take them use conv_kernel)
    const bool halo_ok = !st.gap_finish && halo_input_ok(st) && c.kchunk && c.vec_out && (!c.has_res || c.vec_res) &&
                         (c.mode == M_FLAT || (c.mode == M_ZIGZAG && c.H % 2 == 0 && c.W % 2 == 0)) &&
                         conv_lds_bytes(kHaloCfg, c.mode) <= p.hw.lds_bytes_per_cu;
    // a forced configuration binds the chains it applies to; the others get the planner's choice
    const int force_tile = p.opts.tile >= 1 && p.opts.tile <= kNumTileCfgs ? p.opts.tile
                           : (p.opts.tile == kHaloCfg + 1 || (p.opts.tile >= 7 && p.opts.tile <= 10)) && halo_ok ? kHaloCfg + 1 : 0;
    const int force_halo_bn = p.opts.tile == 7 || p.opts.tile == 9 ? 128 : p.opts.tile == 8 || p.opts.tile == 10 ? 64 : 0;
    const int force_form = p.opts.tile == 7 || p.opts.tile == 8 ? 0 : p.opts.tile == 9 || p.opts.tile == 10 ? 1 : -1;   // 1 = patch-linear
    static const double eff[kNumTileCfgs] = {1.0, 0.85, 0.6, 0.55};
    double best_cost = 1e300;
    int best = -1;
    ConvArgs best_args{};
    for (int cfg = 0; cfg < kNumTileCfgs; ++cfg) {
      if (force_tile > 0 && cfg != force_tile - 1) continue;
      const TileCfg& tc = kTileCfgs[cfg];
      if (conv_lds_bytes(cfg, c.mode) > p.hw.lds_bytes_per_cu) continue;   // parameter split must fit private memory
      if (st.scalar && !conv_cfg_has_scalar_loader(cfg)) continue;
      if (c.dw_w && !conv_cfg_has_dw_prologue(cfg, c.mode)) continue;
      ConvArgs t = c;
      if (c.mode == M_FLAT || c.mode == M_ZIGZAG) {
        t.tiles_m = (c.M_total + tc.bm - 1) / tc.bm;
      } else if (c.mode == M_PATCH) {
        if (!choose_patch(tc.bm, c.pk, c.ps, c.PH, c.PW, &t.pph, &t.ppw)) continue;
        t.patch_h = (t.pph - 1) * c.ps + c.pk;
        t.patch_w = (t.ppw - 1) * c.ps + c.pk;
        t.patches_y = (c.PH + t.pph - 1) / t.pph;
        t.patches_x = (c.PW + t.ppw - 1) / t.ppw;
        t.tiles_m = c.N * t.patches_y * t.patches_x;
      } else {
        t.tiles_m = c.N;
      }
      t.tiles_n = (c.K + tc.bn - 1) / tc.bn;
      t.ntiles = t.tiles_m * t.tiles_n;
      double per_tile = (double)tc.bm * tc.bn / eff[cfg];
      if (c.mode == M_GAP) per_tile *= (double)((c.OH * c.OW + tc.bm - 1) / tc.bm);
      // two workgroups fit on a compute unit; below that, a smaller tile only shortens the critical path
      const double cost = std::max((double)t.ntiles / (2.0 * num_cu), 1.0) * per_tile;
      if (cost < best_cost) { best_cost = cost; best = cfg; best_args = t; }
      if (p.opts.tile == 0) { set_grid(t, cfg); st.cands.push_back(Step::Cand{cfg, t, conv_lds_bytes(cfg, c.mode)}); }
    }
    if (halo_ok && (force_tile == 0 || force_tile == kHaloCfg + 1)) {
      const int step = c.mode == M_ZIGZAG ? 2 : 1;
      const long long rows = (long long)c.N * (c.H + 2);
      ConvArgs t0 = c;
      const double best_fill = choose_halo_tile(c, step, t0) ? 1.0 : 0.0;
      // patch-linear form (pixel-major chains): GEMM row = patch position with pitch TW + 2, two junk rows per patch row;
      // its A fragments are read at the full LDS rate
      ConvArgs tl = c;
      double best_fill_l = 0;
      if (c.mode == M_FLAT) {
        for (int tw = 1; tw <= std::min(c.W, kHaloPitchWide - 2); ++tw) {
          const int pw = tw + 2;
          const int th = std::min(kHaloRows / pw, (kHaloPatchMax - 2) / pw - 2);
          if (th < 1) continue;
          const long long ty = (rows + th - 1) / th, tx = (c.W + tw - 1) / tw;
          const double fill = (double)c.N * c.H * c.W / ((double)ty * tx * kHaloRows);
          if (fill > best_fill_l + 1e-9) { best_fill_l = fill; tl.th = th; tl.tw = tw; tl.tiles_y = (int)ty; tl.tiles_x = (int)tx; }
        }
      }
      for (int form = 0; form < 2; ++form) {
        ConvArgs& t = form == 0 ? t0 : tl;
        if ((form == 0 ? best_fill : best_fill_l) <= 0) continue;
        if (force_form >= 0 && form != force_form && (force_form == 0 || best_fill_l > 0)) continue;   // (zig-zag chains have no patch-linear form)
        t.halo_plin = form;
        t.tiles_m = t.tiles_y * t.tiles_x;
        // one persistent 512-thread workgroup per compute unit walks ceil(tiles / units) tiles.  Measured per-flop
        // rate relative to the 128x128 gather tile: about 3.2x with 128 channels per tile, about 2.6x with 64
        // (three LDS fragment reads per two MFMAs instead of one per MFMA).
        static const int bns[2] = {128, 64};
        static const double rate[2] = {3.2, 2.6};
        for (int v = 0; v < 2; ++v) {
          if (force_halo_bn && bns[v] != force_halo_bn) continue;
          ConvArgs u = t;
          u.halo_bn = bns[v];
          u.tiles_n = (c.K + bns[v] - 1) / bns[v];
          u.ntiles = u.tiles_m * u.tiles_n;
          // Below half a tile per unit the long per-tile pipeline of this kernel (and its 512-thread epilogue) loses
          // to the small gather tiles, which can also split the reduction (measured on the batch-1 networks).
          const bool thin = 2 * u.ntiles < num_cu && force_tile == 0;   // (still a candidate for the tuner when at least 32 tiles)
          // (the patch-linear form measured within +-3 % of the plain one, 6 % faster on 14x14 maps: same model, ties go
          // to the plain form, the tuner decides by measurement)
          const double per_tile = (double)kHaloRows * bns[v] / rate[v];
          const double cost = (double)((u.ntiles + num_cu - 1) / num_cu) * per_tile;
          if (cost < best_cost && !thin) { best_cost = cost; best = kHaloCfg; best_args = u; }
          if (p.opts.tile == 0 && (!thin || u.ntiles >= 32)) { set_grid(u, kHaloCfg); st.cands.push_back(Step::Cand{kHaloCfg, u, conv_lds_bytes(kHaloCfg, c.mode)}); }
        }
      }
    }
    if (best < 0) return fail(XENOS_EUNSUPPORTED, "%s: no tile configuration fits %zu bytes of LDS (or the forced one does not apply)",
                              st.name.c_str(), p.hw.lds_bytes_per_cu);
    c = best_args;
    st.cfg = best;
    set_grid(c, best);
    st.lds = conv_lds_bytes(best, c.mode);
    return XENOS_OK;
  }

  // ---- pack weights of a dense conv / fc in operand order -------------------------------------
  // Csrc = channels of the operator's weights, C = channels the kernel reduces over (>= Csrc, extra ones zero)
  void pack_dense(Step& st, const GOp& o, int Csrc, int C, int R, int S, int K) {
    const int bke = kRowBytes / p.esz;
    const int kred = R * S * C, kred_pad = (kred + bke - 1) / bke * bke;
    const int kout_pad = (K + 127) / 128 * 128;
    st.conv.Kred = kred; st.conv.Kred_pad = kred_pad;
    const size_t bytes = (size_t)kout_pad * kred_pad * p.esz;
    st.w_off = (long long)wpush(nullptr, bytes);
    unsigned char* base = p.wimage.data() + st.w_off;
    memset(base, 0, bytes);
    // source [K][C][R][S] -> destination [K][reduction index]; the reduction index is (r*S+s)*C + c, or, when
    // the channels divide into whole steps, ((c/step)*R*S + r*S + s)*step + c%step so that the R*S taps of
    // one channel chunk are consecutive steps and re-read the same input pixels while they are still cached
    const bool kchunk = C % bke == 0 && R * S > 1 && !st.scalar && !st.fc_stream;
    st.conv.kchunk = kchunk ? 1 : 0;
    // channel of the operator's weights that multiplies channel c of the tensor in memory: the same one, or, behind a
    // folded shuffle of g groups (tensor channel j * m + i is the operator's channel i * g + j), its shuffled position
    const int shg = pack_shuffle_groups, shm = shg ? Csrc / shg : 1;
    auto wch = [&](int c) -> size_t { return shg ? (size_t)(c % shm) * shg + c / shm : (size_t)c; };
    auto kidx = [&](int c, int rs) -> size_t {
      return kchunk ? ((size_t)(c / bke) * R * S + rs) * bke + c % bke : (size_t)rs * C + c;
    };
    if (st.fc_stream) {
      // Weight-streaming kernel: the fragments of a 32-channel block are stored in the order its wavefront loads them,
      // [block][step of 64][k-group of 16][lane = 32 * (half of the k-group) + channel][8 elements], so every load
      // instruction reads 1 KB of consecutive memory and a block's share of the reduction is one sequential stream
      const int nsteps = kred_pad / 64;
      uint16_t* dst = (uint16_t*)base;
      for (int k = 0; k < K; ++k) {
        const float* src = o.weight.data() + (size_t)k * Csrc * R * S;
        for (int c = 0; c < Csrc; ++c)
          for (int rs = 0; rs < R * S; ++rs) {
            const size_t kk = (size_t)rs * C + c;
            const size_t step = kk / 64, g = (kk % 64) / 16, half = (kk % 16) / 8, e = kk % 8;
            dst[(((((size_t)(k / 32) * nsteps + step) * 4 + g) * 64 + half * 32 + k % 32) * 8) + e] = f2bf_host(src[wch(c) * R * S + rs]);
          }
      }
      st.bytes_w = (long long)K * R * S * Csrc * p.esz;
      return;
    }
    for (int k = 0; k < K; ++k) {
      const float* src = o.weight.data() + (size_t)k * Csrc * R * S;
      if (p.dt == DT_BF16) {
        uint16_t* dst = (uint16_t*)base + (size_t)k * kred_pad;
        for (int c = 0; c < Csrc; ++c)
          for (int rs = 0; rs < R * S; ++rs) dst[kidx(c, rs)] = f2bf_host(src[wch(c) * R * S + rs]);
      } else {
        float* dst = (float*)base + (size_t)k * kred_pad;
        for (int c = 0; c < Csrc; ++c)
          for (int rs = 0; rs < R * S; ++rs) dst[kidx(c, rs)] = src[wch(c) * R * S + rs];
      }
    }
    st.bytes_w = (long long)K * R * S * Csrc * p.esz;
  }

  // ---- main pass --------------------------------------------------------------------------------
  xenos_status run() {
    p.dt = p.opts.compute == XENOS_BF16 ? DT_BF16 : DT_F32;
    p.esz = p.dt == DT_BF16 ? 2 : 4;
    p.ce = 16 / p.esz;
    p.zero_off = wpush(nullptr, 256);      // (new bytes of the image are zero)
    build_nodes();
    const int nn = (int)nodes.size();
    tview.assign(nn + 1, -1);
    node_step.assign(nn, -1);
    node_final.assign(nn, 0);
    free_concat.assign(nn, 0);
    ileave.assign(nn, 0);
    alias_shuffle.assign(nn, 0);
    fin_concat.assign(nn, 0);
    fold_shuffle.assign(nn, 0);

    // Channel shuffle as a layout-only link: shuffle(concat(x_0 .. x_{g-1})) with g groups and g equal parts puts channel
    // i of part j at position i * g + j, so the concat buffer is written interleaved and the shuffle moves nothing.  A
    // part that ends a plain dense-convolution chain is stored that way by the chain itself (channel stride g in its
    // epilogue); any other part (the pass-through half of a ShuffleNet unit) is copied into its positions.
    if (p.opts.link >= 2)
      for (int j = 0; j < nn; ++j) {
        if (nodes[j].kind != XENOS_OP_SHUFFLE || j + 1 == out_tid) continue;
        const int t = nodes[j].in[0], g = desc(nodes[j]).groups;
        if (t < 1 || t == out_tid || nodes[t - 1].kind != XENOS_OP_CONCAT || consumers[t].size() != 1 || g < 2) continue;
        const Node& cat = nodes[t - 1];
        if ((int)cat.in.size() != g) continue;
        bool ok = true;
        for (size_t a = 0; a < cat.in.size(); ++a) {
          if (tshape[cat.in[a]].c * g != cat.out.c) ok = false;
          for (size_t b = a + 1; b < cat.in.size(); ++b)
            if (cat.in[a] == cat.in[b]) ok = false;
        }
        if (!ok) continue;
        ileave[t - 1] = g;
        alias_shuffle[j] = 1;
        // Two groups of whole 16-byte channel groups: the part whose plain convolution chain runs last reads the other
        // part (complete by then) in its epilogue and stores both, alternating, with 16-byte stores; nothing else is
        // copied or stored with a stride.
        if (g == 2 && tshape[cat.in[0]].c % p.ce == 0) {
          int best = -1, best_conv = -1;
          for (int a = 0; a < 2; ++a) {
            const int cv = plain_chain_conv(cat.in[a]), other = cat.in[1 - a];
            if (cv < 0 || other < 1 || other == out_tid || other - 1 >= cv) continue;   // the other part must be complete first
            if (cv > best_conv) { best = a; best_conv = cv; }
          }
          if (best >= 0) {
            fin[cat.in[best]] = Fin{t, best, cat.in[1 - best]};
            fin_concat[t - 1] = 1;
            continue;
          }
        }
        for (int a = 0; a < g; ++a)
          if (stores_strided(cat.in[a])) placed[cat.in[a]] = Place{t, a, g};
      }

    // concat realised as channel-offset stores of its producers (Eq. 1: split halves join without a
    // layout transformation)
    if (p.opts.link >= 2)
      for (int i = 0; i < nn; ++i) {
        if (nodes[i].kind != XENOS_OP_CONCAT || ileave[i]) continue;
        const int ctot = nodes[i].out.c;
        bool ok = ctot % p.ce == 0;
        int off = 0;
        for (int t : nodes[i].in) {
          if (t == 0 || t == out_tid || placed.count(t) || fin.count(t) || off % p.ce != 0) ok = false;
          else if (nodes[t - 1].kind == XENOS_OP_CONCAT) ok = false;
          else if (nodes[t - 1].kind == XENOS_OP_SHUFFLE && alias_shuffle[t - 1]) ok = false;   // (its tensor is its concat's buffer)
          off += tshape[t].c;
        }
        for (size_t a = 0; a < nodes[i].in.size(); ++a)
          for (size_t b = a + 1; b < nodes[i].in.size(); ++b)
            if (nodes[i].in[a] == nodes[i].in[b]) ok = false;
        if (!ok) continue;
        free_concat[i] = 1;
        off = 0;
        for (int t : nodes[i].in) { placed[t] = Place{i + 1, off, 1}; off += tshape[t].c; }
      }

    // A shuffle read by dense convolutions only is a permutation of their input channels: the weights are packed in the
    // order of the un-shuffled tensor and the shuffle moves nothing (a layout-only link on the consumer side).
    if (p.opts.link >= 2)
      for (int j = 0; j < nn; ++j) {
        if (nodes[j].kind != XENOS_OP_SHUFFLE || alias_shuffle[j] || j + 1 == out_tid || nodes[j].in[0] < 1 || consumers[j + 1].empty()) continue;
        bool ok = true;
        for (int c : consumers[j + 1]) ok = ok && nodes[c].kind == XENOS_OP_CONV && desc(nodes[c]).groups == 1;
        if (ok) fold_shuffle[j] = 1;
      }

    // graph input
    {
      bool direct = ext_is_internal(p.in) && p.in.c % p.ce == 0;
      bool all_dense = !consumers[0].empty();
      for (int ci : consumers[0]) {
        const Node& nd = nodes[ci];
        if (!(nd.kind == XENOS_OP_CONV && desc(nd).groups == 1)) all_dense = false;
      }
      const int ev = tag(ext_view(p.in, 1), 0);
      tview[0] = ev;
      if (direct) {
        normalise_1x1(p.views[ev]);
        p.views[ev].f32 = 0;
      } else {
        // Otherwise each consumer decides when it is planned.  A first-layer chain whose reduction fits one MFMA
        // pass reads the caller's tensor where it lies (stem kernel); with small inputs any dense convolution
        // gathers from it element-wise (one pass fewer); everything else triggers one import pass.
        in_lazy = true;
        in_all_dense = all_dense;
        in_gather = all_dense && p.in.c <= 8 && (long long)p.in.n * p.in.h * p.in.w < 100000;
      }
    }

    for (int i = 0; i < nn; ++i) {
      if (node_step[i] >= 0) continue;
      xenos_status rc = plan_node(i);
      if (rc != XENOS_OK) return rc;
    }

    if (need_export) {
      Step st;
      st.kind = S_CVT; st.name = "export";
      st.v_in = tview[out_tid];
      st.v_out = tag(ext_view(p.out, 2), out_tid);
      fill_cvt(st);
      add_step(st);
    }
    if (out_tid == 0) return fail(XENOS_EUNSUPPORTED, "graph output is the graph input");
    allocate();
    write_json();
    return XENOS_OK;
  }

  void fill_cvt(Step& st) {
    const View& a = p.views[st.v_in];
    const View& b = p.views[st.v_out];
    CvtArgs& c = st.cvt;
    c.N = a.s.n; c.C = a.s.c; c.Cout = a.s.c; c.H = a.s.h; c.W = a.s.w;
    c.in_sN = a.sN; c.in_sC = a.sK; c.in_sP = a.sP; c.in_f32 = a.f32;
    c.out_sN = b.sN; c.out_sC = b.sK; c.out_sP = b.sP; c.out_f32 = b.f32;
    st.bytes_in = view_bytes(st.v_in);
    st.bytes_out = view_bytes(st.v_out);
  }

  void add_step(Step& st) {
    const int idx = (int)p.steps.size();
    if (st.v_in >= 0) touch(st.v_in, idx);
    if (st.v_in2 >= 0) touch(st.v_in2, idx);
    if (st.v_out >= 0) touch(st.v_out, idx);
    if (st.v_out2 >= 0) touch(st.v_out2, idx);
    p.steps.push_back(st);
  }

  bool available(int tid) const {
    if (tid == 0) return true;
    return node_step[tid - 1] >= 0 && node_final[tid - 1] && tview[tid] >= 0;
  }

  int single_consumer(int tid) const {
    if (tid == out_tid || consumers[tid].size() != 1) return -1;
    return consumers[tid][0];
  }

  // import: convert the graph input to the internal NHWC layout of the compute type.  When only dense
  // convolutions read it (the usual 3-channel image), the channels are zero-padded to a whole 16-byte group so
  // that the first layer runs on the vector loader like every other layer (its padded weights are zero).
  int import_input() {
    const int cpad = in_all_dense ? (p.in.c + p.ce - 1) / p.ce * p.ce : p.in.c;
    const int iv = tag(internal_view(tshape[0], -1, cpad), 0);
    p.views[iv].cphys = cpad;
    Step st;
    st.kind = S_CVT; st.name = "import";
    st.v_in = tview[0]; st.v_out = iv;
    fill_cvt(st);
    st.cvt.Cout = cpad;
    add_step(st);
    tview[0] = iv;
    in_lazy = false;
    return iv;
  }

  xenos_status need_internal_input(int tid, const char* who, int* view) {
    const int v = tview[tid];
    if (v < 0) return fail(XENOS_EINVAL, "%s: input tensor %d is not materialised", who, tid);
    const View& vw = p.views[v];
    if (!vw.internal_nhwc() || vw.f32 != 0 || vw.esz != p.esz) {
      // the graph input reaches an operator that needs the internal layout: import once
      if (tid != 0) return fail(XENOS_EUNSUPPORTED, "%s: tensor %d has no internal layout", who, tid);
      *view = import_input();
      return XENOS_OK;
    }
    *view = v;
    return XENOS_OK;
  }

  // ---- the link pass for one convolution: which operators behind it join its chain (Section 4.1, Table 1) ------
  // conv -> (bias | bn)* -> [add shortcut] -> [relu] -> [max / avg / global pooling]; a depthwise convolution takes no
  // shortcut and no pooling.  Changes nothing in the plan, so the pattern checks of the deeper links may call it for
  // nodes that are planned later.
  struct ChainWalk {
    Affine af;                     // folded scale / shift of the absorbed bias / bn operators (and the convolution's own bias)
    bool relu = false, has_res = false;
    int res_tid = -1, pool_node = -1;
    int cur = 0, last = 0;         // the chain's output tensor and last node
    std::vector<int> absorbed;
  };
  ChainWalk walk_chain(int i) const {
    const Node& nd = nodes[i];
    const GOp& go = g.ops[nd.src];
    const int link = p.opts.link;
    const bool dw = nd.kind == XENOS_OP_CONV && desc(nd).groups != 1;
    ChainWalk w;
    w.af.scale.assign(desc(nd).out_c, 1.0);
    w.af.shift.assign(desc(nd).out_c, 0.0);
    if (!go.bias.empty()) fold_bias(w.af, go.bias);
    w.cur = i + 1; w.last = i;
    int stage = 0;
    while (link >= 1) {
      const int nx = single_consumer(w.cur);
      if (nx < 0 || placed.count(w.cur)) break;
      const Node& nn_ = nodes[nx];
      const GOp& ng = g.ops[nn_.src];
      if ((nn_.kind == XENOS_OP_BIAS || nn_.kind == XENOS_OP_BN) && stage == 0) {
        if (nn_.kind == XENOS_OP_BIAS) fold_bias(w.af, ng.bias); else fold_bn(w.af, ng);
      } else if (nn_.kind == XENOS_OP_ADD && link >= 2 && !dw && stage <= 1) {
        const int other = nn_.in[0] == w.cur ? nn_.in[1] : nn_.in[0];
        if (other == w.cur || !available(other) || other == 0) break;
        const View& ov = p.views[tview[other]];
        if (!ov.internal_nhwc() || ov.f32) break;
        w.has_res = true; w.res_tid = other; stage = 2;
      } else if (nn_.kind == XENOS_OP_RELU && stage <= 2) {
        w.relu = true; stage = 3;
      } else if ((nn_.kind == XENOS_OP_MAXPOOL || nn_.kind == XENOS_OP_AVGPOOL || nn_.kind == XENOS_OP_GLOBAL_AVGPOOL) &&
                 link >= 2 && !dw && (!w.has_res || nn_.kind == XENOS_OP_GLOBAL_AVGPOOL) && stage <= 3) {
        w.pool_node = nx; stage = 4;
      } else {
        break;
      }
      w.absorbed.push_back(nx);
      w.cur = nx + 1; w.last = nx;
      if (stage == 4) break;
    }
    return w;
  }

  // depthwise weights [C][k*k] -> [tap][C] in the compute type; returns the byte offset in the weight image
  long long pack_depthwise(const GOp& go, int C, int taps) {
    const size_t bytes = (size_t)taps * C * p.esz;
    const long long off = (long long)wpush(nullptr, bytes);
    unsigned char* base = p.wimage.data() + off;
    for (int c = 0; c < C; ++c)
      for (int t = 0; t < taps; ++t) {
        const float v = go.weight[(size_t)c * taps + t];
        if (p.dt == DT_BF16) ((uint16_t*)base)[(size_t)t * C + c] = f2bf_host(v);
        else ((float*)base)[(size_t)t * C + c] = v;
      }
    return off;
  }

  // ---- link level 3, pointwise -> depthwise (Section 2.2; Table 1, ConvX -> ConvY) -------------------------------
  // Can the dense convolution node `i` keep its output on chip for the depthwise convolution that consumes it?
  // conv 1x1 / stride 1 / pad 0 -> (bias | bn)* -> [relu] -> depthwise 3x3 / pad 1 / stride 1 or 2 -> (bias | bn)* -> [relu],
  // nothing else reading the tensors in between, whole 16-byte channel groups.  Returns the depthwise node or -1.
  int pwdw_consumer(int i) const {
    if (p.opts.link < 3 || p.opts.tile != 0 || i < 0 || node_step[i] >= 0) return -1;
    const Node& nd = nodes[i];
    if (nd.kind != XENOS_OP_CONV) return -1;
    const xenos_op_desc& d = desc(nd);
    const Shape is = tshape[nd.in[0]];
    if (d.groups != 1 || d.kh != 1 || d.kw != 1 || d.stride_h != 1 || d.pad_h != 0 || nd.in[0] == 0 ||
        is.c % p.ce != 0 || d.out_c % p.ce != 0) return -1;
    const ChainWalk w = walk_chain(i);
    if (w.has_res || w.pool_node >= 0 || w.cur == out_tid || placed.count(w.cur) || fin.count(w.cur)) return -1;
    const int dn = single_consumer(w.cur);
    if (dn < 0 || node_step[dn] >= 0 || nodes[dn].kind != XENOS_OP_CONV) return -1;
    const xenos_op_desc& dd = desc(nodes[dn]);
    if (dd.groups != d.out_c || dd.out_c != d.out_c || dd.kh != 3 || dd.kw != 3 || dd.pad_h != 1 || (dd.stride_h != 1 && dd.stride_h != 2)) return -1;
    const ChainWalk w2 = walk_chain(dn);
    if (fin.count(w2.cur)) return -1;
    auto pl = placed.find(w2.cur);
    if (pl != placed.end() && (pl->second.c_stride != 1 || pl->second.c_off % p.ce != 0)) return -1;   // (16-byte stores only)
    if (w2.cur == out_tid && !ext_is_internal(p.out)) return -1;
    return dn;
  }
  // The pointwise -> depthwise link is taken where the depthwise -> pointwise one (dwpw_kernel, up to 32 channel groups) is
  // no alternative for that depthwise convolution, or where the pointwise convolution behind it can again hand on to a
  // depthwise one, so that a depthwise-separable stack becomes a sequence of pointwise -> depthwise chains (the tensors
  // that reach memory are then the depthwise outputs, the smaller ones of each block).
  bool pwdw_wanted(int i, int dn) const {
    const int C = desc(nodes[dn]).out_c;
    if (C / p.ce > 32) return true;
    const ChainWalk w2 = walk_chain(dn);
    const int nx = placed.count(w2.cur) ? -1 : single_consumer(w2.cur);
    if (nx < 0 || nodes[nx].kind != XENOS_OP_CONV) return true;
    const xenos_op_desc& nd2 = desc(nodes[nx]);
    if (nd2.groups != 1 || nd2.kh != 1 || nd2.kw != 1 || nd2.stride_h != 1 || nd2.pad_h != 0) return true;
    (void)i;
    return pwdw_consumer(nx) >= 0;
  }

  // Tile of depthwise output pixels for a pointwise -> depthwise chain: the GEMM runs over the block positions inside
  // the map in chunks of 64, so the cost of a tile is its chunk count (+ a fixed part); the longest workgroup queue
  // decides.  Two workgroups share a compute unit.
  bool choose_pwdw_tile(ConvArgs& c) const {
    const int s = c.dw_stride, num_cu = std::max(1, p.hw.num_cu);
    const size_t lds_cap = std::min<size_t>(p.hw.lds_bytes_per_cu, 160 * 1024);
    double best = 1e300;
    for (int th = 1; th <= c.OH; ++th)
      for (int tw = 1; tw <= c.OW; ++tw) {
        const int PH = (th - 1) * s + 3, PWd = (tw - 1) * s + 3;
        if (PH * PWd > kPwDwMaxPositions) break;
        if (pwdw_lds_bytes(th, tw, s, p.esz) > lds_cap) break;
        const int ty = (c.OH + th - 1) / th, tx = (c.OW + tw - 1) / tw;
        double total = 0, longest = 0;
        for (int y = 0; y < ty; ++y) {
          const int iy0 = y * th * s - 1, hv = std::min(iy0 + PH, c.H) - std::max(iy0, 0);
          for (int x = 0; x < tx; ++x) {
            const int ix0 = x * tw * s - 1, wv = std::min(ix0 + PWd, c.W) - std::max(ix0, 0);
            const double cost = (hv * wv + 63) / 64 + 0.75;
            total += cost; longest = std::max(longest, cost);
          }
        }
        const double tiles_n = (c.K + kPwDwChannels - 1) / kPwDwChannels;
        // (the second term stands for the traffic of the whole launch, input block and weight slice per tile: among
        // tilings that fit one round it prefers the one with the least recomputation)
        const double all = total * c.N * tiles_n;
        const double t = p.opts.split ? std::max(all / (2.0 * num_cu), longest) + all / (8.0 * num_cu) : total;
        if (t < best - 1e-9) { best = t; c.th = th; c.tw = tw; c.tiles_y = ty; c.tiles_x = tx; }
      }
    return best < 1e300;
  }

  // ---- link level 3, Fire module (Table 1, Conv1x1 -> Conv3x3; Section 4.1 last paragraph) -----------------------
  // squeeze = conv 1x1 / stride 1 / pad 0 (or, over whole reduction steps of input channels, 3x3 / stride 1 / pad 1: Table 1,
  // Conv3x3 -> Conv1x1 and Conv3x3 -> Conv3x3) with at most 64 output channels whose chain output is read by dense convolutions
  // only: one 1x1 / pad 0 and one 3x3 / pad 1 (stride 1) (a Fire module), or one of the two alone (a plain ConvX -> ConvY
  // pair); each a plain chain (bias / bn / relu) that may end in a max-pooling of 2- or 3-wide windows at stride 2 without
  // padding (of a module: the SAME pooling, the one the link pass moved in front of their concat); the outputs take
  // 16-byte stores.
  struct FireMatch { int e[2] = {-1, -1}; };
  bool fire_consumers(int i, FireMatch* fm) const {
    if (p.opts.link < 3 || p.opts.tile != 0 || node_step[i] >= 0) return false;
    const Node& nd = nodes[i];
    if (nd.kind != XENOS_OP_CONV || nd.in[0] == 0) return false;
    const xenos_op_desc& d = desc(nd);
    const Shape is = tshape[nd.in[0]];
    const int S = d.out_c;
    const bool first3 = d.kh == 3 && d.kw == 3 && d.pad_h == 1 && d.pad_w == 1;
    if (d.groups != 1 || d.stride_h != 1 || d.stride_w != 1 || is.c % p.ce != 0 || S > 64 || (S * p.esz) % 32 != 0) return false;
    if (!first3 && (d.kh != 1 || d.kw != 1 || d.pad_h != 0 || d.pad_w != 0)) return false;
    // (a 3x3 first convolution reads the taps of a chunk of input channels in consecutive steps: whole chunks only)
    if (first3 && (std::max(is.c, p.views[tview[nd.in[0]]].cphys) % (kRowBytes / p.esz) != 0 || is.h > 0xffff || is.w > 0xffff)) return false;
    // (fp32 at large batch: the module as three chains on the big GEMM tiles is faster than one chain whose squeeze halo is
    // recomputed at the fp32 MFMA rate; measured on the SqueezeNet graph at batch 32, 0.67 against 0.74 ms)
    if (p.dt == DT_F32 && (long long)is.n * is.h * is.w > 4096) return false;
    const ChainWalk w = walk_chain(i);
    if (w.has_res || w.pool_node >= 0 || w.cur == out_tid || placed.count(w.cur) || fin.count(w.cur) || (consumers[w.cur].size() != 2 && consumers[w.cur].size() != 1)) return false;
    int pool_src = -2;
    for (int c : consumers[w.cur]) {
      const Node& en = nodes[c];
      if (en.kind != XENOS_OP_CONV || node_step[c] >= 0 || en.in[0] != w.cur) return false;
      const xenos_op_desc& ed = desc(en);
      if (ed.groups != 1 || ed.stride_h != 1 || ed.out_c % p.ce != 0) return false;
      const int which = ed.kh == 1 && ed.kw == 1 && ed.pad_h == 0 ? 0 : ed.kh == 3 && ed.kw == 3 && ed.pad_h == 1 ? 1 : -1;
      if (which < 0 || fm->e[which] >= 0) return false;
      const ChainWalk we = walk_chain(c);
      if (we.has_res || fin.count(we.cur)) return false;
      int ps = -1;
      if (we.pool_node >= 0) {
        const xenos_op_desc& pd = desc(nodes[we.pool_node]);
        if (pd.kind != XENOS_OP_MAXPOOL || pd.kh != pd.kw || (pd.kh != 2 && pd.kh != 3) || pd.stride_h != 2 || pd.pad_h != 0) return false;
        ps = nodes[we.pool_node].src;
      }
      if (pool_src != -2 && ps != pool_src) return false;           // both parts pooled by the same operator, or neither
      pool_src = ps;
      auto pl = placed.find(we.cur);
      if (pl != placed.end() && (pl->second.c_stride != 1 || pl->second.c_off % p.ce != 0)) return false;
      if (we.cur == out_tid && !ext_is_internal(p.out)) return false;
      fm->e[which] = c;
    }
    if (fm->e[0] < 0 && fm->e[1] < 0) return false;
    const int pk = pool_src >= 0 ? g.ops[pool_src].d.kh : 0;
    return fire_lds_bytes(pk ? pk : 1, pk ? pk : 1, S, p.esz, pk ? 1 : 0, fm->e[1] >= 0 ? 1 : 0) <= std::min<size_t>(p.hw.lds_bytes_per_cu, 160 * 1024);
  }

  // Tile (output pixels, or pooling windows) and number of channel shares of a Fire-module chain.  A workgroup's time in
  // microseconds, from timestamps taken inside the kernel at its phase boundaries (bf16, batch 1): 1.4 to start, the
  // squeeze GEMM of its clipped block 1.0 + 0.35 per chunk of 64 positions and reduction step, and for every expand
  // tile of its share the weight copy (0.7 + 0.15 per 4 KB), the GEMM (0.5 + 0.028 per tap and k-group, per chunk of 64
  // pixels) and 0.9 for epilogue and stores (+ 1.5 with a linked pooling): at batch 1 these fixed latencies, not the
  // MFMA work, are the time of a module.  The longest workgroup decides, or the sum of all over the units' slots.
  bool choose_fire_tile(ConvArgs& c) const {
    const int num_cu = std::max(1, p.hw.num_cu);
    const size_t lds_cap = std::min<size_t>(p.hw.lds_bytes_per_cu, 160 * 1024);
    const bool pool = c.pool != POOL_NONE;
    const int S = c.K, kgs = S * p.esz / 32, nsteps = c.Kred_pad / (kRowBytes / p.esz);
    const int nt[2] = {(c.fire_E[0] + 63) / 64, (c.fire_E[1] + 63) / 64};
    const int ring = c.fire_E[1] > 0 ? 1 : 0;                      // halo of the first convolution's block
    const int YH = pool ? c.PH : c.H, XW = pool ? c.PW : c.W;      // extent of the tile grid (windows or pixels)
    double best = 1e300;
    for (int th = 1; th <= YH; ++th)
      for (int tw = 1; tw <= XW; ++tw) {
        const int CH = pool ? (th - 1) * c.ps + c.pk : th, CW = pool ? (tw - 1) * c.ps + c.pk : tw;
        if ((CH + 2 * ring) * (CW + 2 * ring) > kFireMaxPositions) break;
        const size_t lds = fire_lds_bytes(CH, CW, S, p.esz, pool ? 1 : 0, ring);
        if (lds > lds_cap) break;
        const int occ = 2 * lds <= lds_cap ? 2 : 1;
        const int ty = (YH + th - 1) / th, tx = (XW + tw - 1) / tw;
        const double px_chunks = (CH * CW + 63) / 64;
        double sq_total = 0, sq_longest = 0;
        for (int y = 0; y < ty; ++y) {
          const int iy0 = (pool ? y * th * c.ps : y * th) - ring, hv = std::min(iy0 + CH + 2 * ring, c.H) - std::max(iy0, 0);
          for (int x = 0; x < tx; ++x) {
            const int ix0 = (pool ? x * tw * c.ps : x * tw) - ring, wv = std::min(ix0 + CW + 2 * ring, c.W) - std::max(ix0, 0);
            const double cost = 1.0 + ((hv * wv + 63) / 64) * (double)nsteps * (p.dt == DT_BF16 ? 0.35 : 0.5);
            sq_total += cost; sq_longest = std::max(sq_longest, cost);
          }
        }
        for (int shares = 1; shares <= std::max(nt[0], nt[1]); ++shares) {
          // share z takes the expand tiles z, z + shares, ... of each part
          double ex_total = 0, ex_longest = 0;
          for (int z = 0; z < shares; ++z) {
            double e = 0;
            for (int wch = 0; wch < 2; ++wch) {
              const int taps = wch ? 9 : 1;
              const double copy = 0.7 + 0.15 * (64.0 * taps * S * p.esz / 4096.0);
              const double gemm = px_chunks * (0.5 + (p.dt == DT_BF16 ? 0.028 : 0.11) * taps * kgs);
              e += ((nt[wch] - z + shares - 1) / shares) * (copy + gemm + 0.9 + (pool ? 1.5 : 0.0));
            }
            ex_total += e; ex_longest = std::max(ex_longest, e);
          }
          const double wgs = (double)shares * ty * tx * c.N;
          const double all = ((double)shares * sq_total + (double)ty * tx * ex_total) * c.N + 1.4 * wgs;
          const double longest = 1.4 + sq_longest + ex_longest;
          const double t = p.opts.split ? std::max(all / ((double)occ * num_cu), longest) + all / (8.0 * num_cu) : all;
          if (t < best - 1e-9) {
            best = t;
            if (pool) { c.pph = th; c.ppw = tw; c.th = CH; c.tw = CW; } else { c.th = th; c.tw = tw; }
            c.tiles_y = ty; c.tiles_x = tx; c.tiles_n = shares;
          }
        }
      }
    return best < 1e300;
  }

  xenos_status plan_fire(int i, const ChainWalk& w, const FireMatch& fm) {
    const Node& nd = nodes[i];
    const GOp& go = g.ops[nd.src];
    const Shape is = tshape[nd.in[0]];
    const int S = desc(nd).out_c;
    Step st;
    st.kind = S_CONV;
    st.name = std::string("op") + std::to_string(nd.src);
    st.ops.push_back(nd.src);
    for (int ab : w.absorbed) st.ops.push_back(nodes[ab].src);
    st.v_in = tview[nd.in[0]];
    const View iv = p.views[st.v_in];
    ConvArgs& a = st.conv;
    a.N = is.n; a.C = std::max(is.c, iv.cphys); a.H = is.h; a.W = is.w; a.K = S;
    const int R1 = desc(nd).kh;                                    // 1, or 3 (pad 1)
    a.R = R1; a.S = R1; a.stride = 1; a.pad = R1 / 2; a.OH = is.h; a.OW = is.w; a.PH = is.h; a.PW = is.w;
    a.in_sN = iv.sN; a.in_sH = iv.sP * is.w; a.in_sW = iv.sP;
    a.relu = w.relu; a.mode = M_FLAT; a.pool = POOL_NONE; a.fire = 1;
    pack_dense(st, go, is.c, a.C, R1, R1, S);
    if (R1 == 3 && !a.kchunk) return fail(XENOS_EUNSUPPORTED, "%s: 3x3 weights of a linked pair are not packed by channel chunk", st.name.c_str());
    push_affine(w.af, (S + 127) / 128 * 128, &st.scale_off, &st.shift_off);
    const int sidx = (int)p.steps.size();
    node_step[i] = sidx;
    for (int ab : w.absorbed) node_step[ab] = sidx;
    st.flops = 2.0 * is.n * is.h * is.w * (double)S * is.c * R1 * R1;
    for (int which = 0; which < 2; ++which) {
      const int en = fm.e[which];
      if (en < 0) { a.fire_E[which] = 0; a.fire_relu[which] = 0; continue; }   // (a pair: the module's other part does not exist)
      const GOp& eg = g.ops[nodes[en].src];
      const int E = desc(nodes[en]).out_c, taps = which ? 9 : 1, Epad = (E + 63) / 64 * 64;
      const ChainWalk we = walk_chain(en);
      st.ops.push_back(nodes[en].src);
      for (int ab : we.absorbed) st.ops.push_back(nodes[ab].src);
      // weights [E][S][kh][kw] -> [E padded to 64][tap][S] in the compute type
      const size_t bytes = (size_t)Epad * taps * S * p.esz;
      st.fire_w_off[which] = (long long)wpush(nullptr, bytes);
      unsigned char* base = p.wimage.data() + st.fire_w_off[which];
      memset(base, 0, bytes);
      for (int k = 0; k < E; ++k)
        for (int c = 0; c < S; ++c)
          for (int t = 0; t < taps; ++t) {
            const float v = eg.weight[((size_t)k * S + c) * taps + t];
            const size_t o = ((size_t)k * taps + t) * S + c;
            if (p.dt == DT_BF16) ((uint16_t*)base)[o] = f2bf_host(v); else ((float*)base)[o] = v;
          }
      push_affine(we.af, Epad, &st.fire_scale_off[which], &st.fire_shift_off[which]);
      a.fire_E[which] = E; a.fire_relu[which] = we.relu;
      if (we.pool_node >= 0) {
        const xenos_op_desc& pd = desc(nodes[we.pool_node]);
        const Shape ps = tshape[we.pool_node + 1];
        a.pool = POOL_MAX; a.pk = pd.kh; a.ps = pd.stride_h; a.pp = 0; a.PH = ps.h; a.PW = ps.w;
      }
      const int ov = out_view_for(we.cur, true);
      if (which == 0 || fm.e[0] < 0) st.v_out = ov;
      if (which == 1) st.v_out2 = ov;
      const View& o = p.views[ov];
      if (o.sK != 1 || o.f32 || o.esz != p.esz || o.off % p.ce != 0 || o.sP % p.ce != 0 || o.sN % p.ce != 0)
        return fail(XENOS_EUNSUPPORTED, "%s: output of the Fire-module chain is not aligned", st.name.c_str());
      a.fire_sN[which] = o.sN; a.fire_sP[which] = o.sP;
      if (which == 0 || fm.e[0] < 0) { a.out_sN = o.sN; a.out_sP = o.sP; a.out_sK = 1; a.vec_out = 1; }
      node_step[en] = sidx;
      for (int ab : we.absorbed) node_step[ab] = sidx;
      node_final[we.last] = 1;
      const Shape es = tshape[en + 1];
      st.flops += 2.0 * es.n * es.h * es.w * (double)E * taps * S;
      st.bytes_w += (long long)E * taps * S * p.esz;
      st.bytes_out += view_bytes(ov);
    }
    if (!choose_fire_tile(a)) return fail(XENOS_EUNSUPPORTED, "%s: no tile of the Fire-module kernel fits", st.name.c_str());
    a.M_total = a.N * a.H * a.W;
    a.tiles_m = a.N * a.tiles_y * a.tiles_x;
    a.ntiles = a.tiles_m * a.tiles_n;
    a.xcd_m = 8;
    a.grid = p.opts.split ? std::max(1, std::min(a.ntiles, 4 * std::max(1, p.hw.num_cu))) : 1;
    st.cfg = kFireCfg;
    st.lds = fire_lds_bytes(a.th, a.tw, S, p.esz, a.pool != POOL_NONE ? 1 : 0, a.fire_E[1] > 0 ? 1 : 0);
    st.bytes_in = view_bytes(st.v_in);
    add_step(st);
    return XENOS_OK;
  }

  xenos_status plan_node(int i) {
    const int k = nodes[i].kind;
    return k == XENOS_OP_CONV || k == XENOS_OP_FC || k == XENOS_OP_MATMUL ? plan_conv(i) : plan_standalone(i);
  }

  // Plans the chain that convolution / fully connected node `i` starts (and, at link level 3, the convolution it hands
  // its output to on chip).
  xenos_status plan_conv(int i) {
    const Node& nd = nodes[i];
    const xenos_op_desc& d = desc(nd);
    const GOp& go = g.ops[nd.src];
    const int link = p.opts.link;
    const Shape is = tshape[nd.in[0]];
    Step st;
    st.name = std::string("op") + std::to_string(nd.src);
    st.ops.push_back(nd.src);
    auto finish = [&](int, int out_tensor, bool is_conv) { st.v_out = out_view_for(out_tensor, is_conv); };

    {
      // (a matmul is a fully connected operator over a 1x1 map: its rows are the images)
      const bool is_fc = nd.kind == XENOS_OP_FC || nd.kind == XENOS_OP_MATMUL;
      const bool dw = !is_fc && d.groups != 1;
      const int K = d.out_c;
      if (dw && (d.groups != is.c || K != is.c)) return fail(XENOS_EUNSUPPORTED, "%s: only groups == 1 or depthwise (groups == C == out_c)", st.name.c_str());
      if (dw && is.c % p.ce != 0) return fail(XENOS_EUNSUPPORTED, "%s: depthwise channels must be a multiple of %d", st.name.c_str(), p.ce);
      ChainWalk walk = walk_chain(i);
      Affine& af = walk.af;
      bool relu = walk.relu, has_res = walk.has_res;
      int res_tid = walk.res_tid, pool_node = walk.pool_node;
      int cur = walk.cur, last = walk.last;
      std::vector<int>& absorbed = walk.absorbed;
      (void)res_tid;
      // A first layer that can read the graph input in place (stem kernel) does so; that kernel has no pooling
      // epilogue, so a pooling that follows it runs as its own pass over the (NHWC, compute-type) result.  Measured
      // on the 7x7/2 + 3x3/2-pool and 3x3/2 + 3x3/2-pool first layers, the two passes take about a third of the time
      // of import + a pooled gather chain.
      bool stem = false, stem_lds = false;
      // (the gather form takes reductions up to kStemRed elements, the LDS-staged form up to 4 channels x 7 x 7 taps)
      if (!dw && !is_fc && nd.in[0] == 0 && in_lazy && link >= 2 && !has_res && (is.c * d.kh * d.kw <= kStemRed || (is.c <= 4 && d.kh <= 7 && d.kw <= 7)) &&
          // (32 or 64 output channels, or up to a quarter fewer: the kernels compute the padded count)
          K <= 64 && K % p.ce == 0 && 4 * ((K <= 32 ? 32 : 64) - K) <= (K <= 32 ? 32 : 64) && is.h <= 8192 &&
          conv_lds_bytes(kStemCfg, M_FLAT) <= p.hw.lds_bytes_per_cu && (p.opts.tile == 0 || p.opts.tile == kStemCfg + 1)) {
        // l2 = last node of the chain without its pooling, c2 = that node's output tensor
        const int l2 = pool_node < 0 ? last : absorbed.size() >= 2 ? absorbed[absorbed.size() - 2] : i;
        const int c2 = l2 + 1;
        // The kernel that stages the input block in LDS (bf16 path, fp32 NCHW input with unit stride along W, at most 4
        // channels, square kernel of 4x4 to 7x7, stride 1 or 2; measured at batch 32: 7x7 / 2 on 224x224 0.043 ms against
        // 0.077 ms for the gather form, while 3x3 kernels, 9 gathers per pixel and channel, are faster on the gather form)
        // takes a linked max-pooling of 2 or 3 wide windows at stride 2: 3 x 8 windows per tile, their convolution block
        // recomputed per tile.
        const View& gv = p.views[tview[0]];
        stem_lds = p.dt == DT_BF16 && p.opts.tile == 0 && is.c <= 4 && d.kh == d.kw && d.kh >= 3 && d.kh <= 7 && d.stride_h == d.stride_w &&
                   (d.stride_h == 1 || d.stride_h == 2) && d.pad_h == d.pad_w && d.pad_h <= d.kh && gv.f32 && gv.sP == 1 &&
                   ((kStemLdsTh - 1) * d.stride_h + d.kh) * ((kStemLdsTw - 1) * d.stride_h + d.kw) <= stem_lds_in_positions(d.kh * d.kw);
        bool keep_pool = false;
        if (stem_lds && pool_node >= 0 && !placed.count(cur) && cur != out_tid) {
          const xenos_op_desc& pd = desc(nodes[pool_node]);
          const int chh = (kStemLdsPph - 1) * 2 + pd.kh, cww = (kStemLdsPpw - 1) * 2 + pd.kw;
          keep_pool = pd.kind == XENOS_OP_MAXPOOL && pd.kh == pd.kw && (pd.kh == 2 || pd.kh == 3) && pd.stride_h == 2 && pd.stride_w == 2 &&
                      pd.pad_h == pd.pad_w && pd.pad_h >= 0 && pd.pad_h <= 1 && chh * cww <= kStemLdsTh * kStemLdsTw &&
                      ((chh - 1) * d.stride_h + d.kh) * ((cww - 1) * d.stride_h + d.kw) <= stem_lds_in_positions(d.kh * d.kw);
        }
        // (a 3x3 layer takes the LDS-staged form only for its linked pooling: one launch for two, the same time at batch 32;
        // without pooling the gather form is faster)
        if (stem_lds && d.kh < 4 && !keep_pool) stem_lds = false;
        // (a padded channel count only where the chain stays as linked as the general kernel would have it)
        const bool padded = K != 32 && K != 64;
        if ((stem_lds || is.c * d.kh * d.kw <= kStemRed) && (keep_pool || (c2 != out_tid && !placed.count(c2) && !(padded && pool_node >= 0)))) {
          stem = true;
          if (pool_node >= 0 && !keep_pool) { absorbed.pop_back(); pool_node = -1; cur = c2; last = l2; }
        } else {
          stem_lds = false;
        }
      }
      for (int a : absorbed) st.ops.push_back(nodes[a].src);

      // link level 3, ConvX -> ConvY: a 3x3 first layer whose only consumer is a 3x3 convolution of the same 64 channels
      // is produced tile by tile (halo recomputed) inside that convolution's kernel and never written to memory
      if (stem && link >= 3 && p.dt == DT_BF16 && p.opts.tile == 0 && K == kPairChannels && is.c <= 4 && d.kh == 3 && d.kw == 3 &&
          d.stride_h == 1 && d.stride_w == 1 && d.pad_h == 1 && d.pad_w == 1 && pool_node < 0 && !placed.count(cur) && cur != out_tid) {
        const View& gv = p.views[tview[0]];
        const int nx = single_consumer(cur);
        if (gv.f32 && gv.sP == 1 && nx >= 0 && pair_consumer_ok(nx)) {
          std::vector<uint16_t> w1((size_t)kPairChannels * kPairRed, 0);
          for (int k = 0; k < K; ++k)
            for (int c = 0; c < is.c; ++c)
              for (int t = 0; t < 9; ++t) w1[(size_t)k * kPairRed + t * 4 + c] = f2bf_host(go.weight[((size_t)k * is.c + c) * 9 + t]);
          pairpro = PairPro{};
          pairpro.active = true; pairpro.ops = st.ops; pairpro.relu = relu;
          pairpro.w_off = (long long)wpush(w1.data(), w1.size() * 2);
          push_affine(af, kPairChannels, &pairpro.scale_off, &pairpro.shift_off);
          pairpro.flops = 2.0 * is.n * is.h * is.w * (double)K * 9 * is.c;
          pairpro.bytes_w = (long long)K * 9 * is.c * 2;
          const int mark = (int)p.steps.size();
          node_step[i] = mark;
          for (int a : absorbed) node_step[a] = mark;
          return plan_node(nx);
        }
      }

      if (dw) {
        int vin;
        xenos_status rc = need_internal_input(nd.in[0], st.name.c_str(), &vin);
        if (rc != XENOS_OK) return rc;
        // link level 3: depthwise -> pointwise.  The depthwise result is produced tile by tile inside the
        // pointwise kernel (as its A operand) and never written to memory.
        const int pw = link >= 3 && !placed.count(cur) ? single_consumer(cur) : -1;
        // (a pointwise chain that stores with a channel stride, a part of a shuffled concat of more than two groups, has no
        // 16-byte stores, which the depthwise-panel kernel needs; the element-wise form of the linked pair is slower than
        // two chains.  The chain that finishes a two-group shuffle stores whole groups and can take the depthwise.)
        // (nor one that links a window pooling: the kernels with a depthwise producer enumerate pixel-major rows)
        if (pw >= 0 && d.kh == d.kw && nodes[pw].kind == XENOS_OP_CONV && !chain_stores_strided(pw) && !chain_links_window_pool(pw)) {
          const xenos_op_desc& pd = desc(nodes[pw]);
          // Every workgroup of the pointwise chain recomputes the depthwise result of its 64 pixels for all input
          // channels; beyond 32 channel groups per pixel (8 pixels per thread) that serial work costs more than the
          // saved pass (measured on MobileNet, batch 1: pairs up to 256 channels gain 5-11 us each, wider ones lose 6).
          // (and a pointwise convolution that will hand its own output to the NEXT depthwise convolution on chip keeps this
          // one out: the stack then runs as pointwise -> depthwise chains, see pwdw_wanted)
          const int next_dw = pwdw_consumer(pw);
          if (pd.groups == 1 && pd.kh == 1 && pd.kw == 1 && pd.stride_h == 1 && pd.pad_h == 0 && node_step[pw] < 0 && p.opts.tile == 0 &&
              is.c / p.ce <= 32 && !(next_dw >= 0 && pwdw_wanted(pw, next_dw))) {
            const int taps = d.kh * d.kw;
            const size_t bytes = (size_t)taps * is.c * p.esz;
            dwpro = DwPro{};
            dwpro.active = true; dwpro.v_in = vin; dwpro.ops = st.ops;
            dwpro.w_off = pack_depthwise(go, is.c, taps);
            push_affine(af, is.c, &dwpro.scale_off, &dwpro.shift_off);
            dwpro.k = d.kh; dwpro.stride = d.stride_h; dwpro.pad = d.pad_h; dwpro.H = is.h; dwpro.W = is.w; dwpro.relu = relu;
            dwpro.flops = 2.0 * is.n * tshape[i + 1].h * tshape[i + 1].w * is.c * taps;
            dwpro.bytes_w = (long long)bytes;
            const int mark = (int)p.steps.size();
            node_step[i] = mark;
            for (int a : absorbed) node_step[a] = mark;
            return plan_node(pw);
          }
        }
        st.kind = S_DW;
        st.v_in = vin;
        finish(last, cur, false);
        const View& iv = p.views[st.v_in];
        const View& ov = p.views[st.v_out];
        if (!ov.internal_nhwc() || ov.f32) return fail(XENOS_EUNSUPPORTED, "%s: depthwise output must be internal", st.name.c_str());
        DwArgs& a = st.dw;
        const Shape os = tshape[i + 1];
        a.N = is.n; a.C = is.c; a.H = is.h; a.W = is.w; a.R = d.kh; a.S = d.kw; a.stride = d.stride_h; a.pad = d.pad_h;
        a.OH = os.h; a.OW = os.w; a.in_sN = iv.sN; a.in_sP = iv.sP; a.out_sN = ov.sN; a.out_sP = ov.sP; a.relu = relu;
        a.total_vec = (long long)a.N * a.OH * a.OW * (a.C / p.ce);
        // weights [R*S][C]
        const int taps = d.kh * d.kw;
        const size_t bytes = (size_t)taps * is.c * p.esz;
        st.w_off = pack_depthwise(go, is.c, taps);
        push_affine(af, is.c, &st.scale_off, &st.shift_off);
        st.flops = 2.0 * a.N * a.OH * a.OW * a.C * taps;
        st.bytes_in = view_bytes(st.v_in); st.bytes_w = (long long)bytes; st.bytes_out = view_bytes(st.v_out);
      } else {
        if (!dwpro.active && !pairpro.active && !is_fc && !stem) {
          FireMatch fm;
          if (fire_consumers(i, &fm)) {
            const View& iv0 = p.views[tview[nd.in[0]]];
            if (iv0.internal_nhwc() && !iv0.f32 && iv0.esz == p.esz && iv0.off % p.ce == 0 && iv0.sP % p.ce == 0 && iv0.sN % p.ce == 0)
              return plan_fire(i, walk, fm);
          }
          const int dn = pwdw_consumer(i);
          if (dn >= 0 && pwdw_wanted(i, dn)) {
            const View& iv0 = p.views[tview[nd.in[0]]];
            if (iv0.internal_nhwc() && !iv0.f32 && iv0.esz == p.esz && iv0.off % p.ce == 0 && iv0.sP % p.ce == 0 && iv0.sN % p.ce == 0)
              return plan_pwdw(i, walk, dn);
          }
        }
        st.kind = S_CONV;
        const bool from_dw = dwpro.active;
        const DwPro pro = dwpro;
        dwpro.active = false;
        const bool from_pair = pairpro.active;
        const PairPro ppro = pairpro;
        pairpro.active = false;
        if (!from_dw && nd.in[0] == 0 && in_lazy) {
          st.stem = stem;
          if (!st.stem && !in_gather) import_input();
          st.stem_lds = st.stem && stem_lds;
        }
        const int vin = from_dw ? pro.v_in : from_pair ? tview[0] : tview[nd.in[0]];
        if (vin < 0) return fail(XENOS_EINVAL, "%s: input not materialised", st.name.c_str());
        st.v_in = vin;
        if (from_dw) st.ops.insert(st.ops.begin(), pro.ops.begin(), pro.ops.end());
        if (from_pair) st.ops.insert(st.ops.begin(), ppro.ops.begin(), ppro.ops.end());
        const View& iv = p.views[vin];
        ConvArgs& a = st.conv;
        // padding channels multiply zero weights (not behind a linked depthwise producer: it has no weights for them)
        a.N = is.n; a.C = from_dw ? is.c : std::max(is.c, iv.cphys); a.H = is.h; a.W = is.w;
        a.K = K;
        if (is_fc) { a.R = is.h; a.S = is.w; a.stride = 1; a.pad = 0; a.OH = 1; a.OW = 1; }
        else { a.R = d.kh; a.S = d.kw; a.stride = d.stride_h; a.pad = d.pad_h; a.OH = tshape[i + 1].h; a.OW = tshape[i + 1].w; }
        st.scalar = !(iv.internal_nhwc() && !iv.f32 && iv.esz == p.esz && a.C % p.ce == 0 && iv.off % p.ce == 0 && iv.sP % p.ce == 0);
        a.in_sN = iv.sN; a.in_sH = iv.sP * is.w; a.in_sW = iv.sP; a.in_f32 = iv.f32;
        if (from_dw) {
          st.scalar = 0;
          st.dw_w_off = pro.w_off; st.dw_scale_off = pro.scale_off; st.dw_shift_off = pro.shift_off;
          a.dw_k = pro.k; a.dw_stride = pro.stride; a.dw_pad = pro.pad; a.dw_H = pro.H; a.dw_W = pro.W; a.dw_relu = pro.relu;
          a.dw_sN = iv.sN; a.dw_sP = iv.sP;
          a.dw_w = (const void*)1;           // marks the chain for the split planner; patched at launch
        }
        // The first-layer kernels compute 32 or 64 channels: another channel count (24 in the ShuffleNet graph) is padded
        // with zero weights, and the output tensor gets the padded channel pitch (its consumers read the first K).
        const int Kk = st.stem ? (K <= 32 ? 32 : 64) : K;
        a.K = Kk;
        if (Kk != K) {
          if (tview[cur] >= 0 || placed.count(cur) || cur == out_tid) return fail(XENOS_EUNSUPPORTED, "%s: padded first layer needs a tensor of its own", st.name.c_str());
          tview[cur] = tag(internal_view(tshape[cur], -1, Kk), cur);
          p.views[tview[cur]].cphys = Kk;
        }
        if (st.stem_lds) {
          // weights [K][steps * 16] with reduction slot = tap * 4 + channel (4 taps per MFMA step of 16)
          const int taps = d.kh * d.kw, nstep = taps <= 12 ? 3 : taps <= 28 ? 7 : 13;
          std::vector<uint16_t> ws((size_t)Kk * nstep * 16, 0);
          for (int k = 0; k < K; ++k)
            for (int c = 0; c < is.c; ++c)
              for (int t = 0; t < taps; ++t) ws[(size_t)k * nstep * 16 + t * 4 + c] = f2bf_host(go.weight[((size_t)k * is.c + c) * taps + t]);
          st.dw_w_off = (long long)wpush(ws.data(), ws.size() * 2);
          a.pair_C = is.c; a.pair_sN = iv.sN; a.pair_sC = iv.sK; a.pair_sH = iv.sP * is.w;
        }
        if (from_pair) {
          // `in` is the caller's tensor (fp32, unit stride along W); C, H, W describe the intermediate tensor
          st.scalar = 0;
          a.C = is.c;
          a.pair = 1; a.pair_C = p.in.c; a.pair_sN = iv.sN; a.pair_sC = iv.sK; a.pair_sH = iv.sP * is.w;
          st.dw_w_off = ppro.w_off; st.dw_scale_off = ppro.scale_off; st.dw_shift_off = ppro.shift_off;
          a.dw_relu = ppro.relu;
        }
        a.relu = relu; a.has_res = has_res;
        if (has_res) {
          st.v_in2 = tview[res_tid];
          a.res_sN = p.views[st.v_in2].sN; a.res_sP = p.views[st.v_in2].sP;
        }
        const auto fit = fin.find(cur);
        if (fit != fin.end()) {
          // this chain finishes a two-group shuffle: the other part of the concat comes in where a shortcut would
          const int other = fit->second.other;
          if (has_res || pool_node >= 0 || from_pair || is_fc || !available(other))
            return fail(XENOS_EUNSUPPORTED, "%s: cannot finish the channel shuffle of its concat", st.name.c_str());
          xenos_status rc = need_internal_input(other, st.name.c_str(), &st.v_in2);
          if (rc != XENOS_OK) return rc;
          const View& rv = p.views[st.v_in2];
          if (K % p.ce || rv.off % p.ce || rv.sP % p.ce || rv.sN % p.ce || rv.sK != 1)
            return fail(XENOS_EUNSUPPORTED, "%s: the other half of its shuffled concat is not aligned", st.name.c_str());
          a.res_sN = rv.sN; a.res_sP = rv.sP;
          a.ileave = fit->second.pos + 1;
        }
        a.pool = POOL_NONE; a.mode = M_FLAT;
        a.PH = a.OH; a.PW = a.OW;
        if (pool_node >= 0) {
          const xenos_op_desc& pd = desc(nodes[pool_node]);
          const Shape ps = tshape[pool_node + 1];
          a.PH = ps.h; a.PW = ps.w;
          if (pd.kind == XENOS_OP_GLOBAL_AVGPOOL) { a.pool = POOL_GAP; a.mode = M_GAP; }
          else {
            a.pool = pd.kind == XENOS_OP_MAXPOOL ? POOL_MAX : POOL_AVG;
            a.pk = pd.kh; a.ps = pd.stride_h; a.pp = pd.pad_h; a.cip = pd.count_include_pad;
            a.mode = (a.pk == 2 && a.ps == 2 && a.pp == 0 && 2 * a.PH <= a.OH && 2 * a.PW <= a.OW) ? M_ZIGZAG : M_PATCH;
          }
        }
        // With few images the one-workgroup-per-(image, channel tile) form of the linked global average leaves the chip
        // idle and walks the whole reduction serially; the chain then runs as a pixel-major convolution whose reduction
        // is split across workgroups, and the summing pass applies the epilogue and averages (same single chain of
        // operators, two launches).
        // (a linked depthwise producer needs the depthwise-panel kernel for this, which takes whole channel groups)
        const bool dw_panel_fits = from_dw && a.C % p.ce == 0 && K % p.ce == 0 && !has_res &&
                                   dwpw_lds_bytes(kRowBytes / p.esz, p.esz) <= std::min<size_t>(p.hw.lds_bytes_per_cu, 160 * 1024);
        if (a.mode == M_GAP && p.opts.split && (!from_dw || dw_panel_fits) && 2 * a.N * ((K + 63) / 64) <= std::max(1, p.hw.num_cu) &&
            p.opts.tile == 0) {
          st.gap_finish = 1;
          a.mode = M_FLAT; a.pool = POOL_NONE;
        }
        // a 3x3 layer on a small map: reduction shared out inside the halo kernel (a linked global average then moves
        // to the summing pass as above)
        HaloSplit hsplit;
        if (!from_dw && !from_pair && !is_fc && !st.stem && !a.ileave && (a.mode == M_FLAT || a.mode == M_GAP)) hsplit = choose_halo_split(st);
        if (hsplit.ks >= 2 && a.mode == M_GAP) {
          st.gap_finish = 1;
          a.mode = M_FLAT; a.pool = POOL_NONE;
        }
        a.M_total = a.mode == M_FLAT ? a.N * a.OH * a.OW : a.mode == M_ZIGZAG ? a.N * a.PH * a.PW * 4 : a.OH * a.OW;
        // A fully connected chain over at most 32 images streams its weights once: the kernel made for that keeps many
        // loads in flight per unit and shares the reduction out over workgroups (the summing pass finishes the chain)
        st.fc_stream = !a.ileave && p.dt == DT_BF16 && p.opts.split && p.opts.tile == 0 && !from_dw && !from_pair && a.mode == M_FLAT && !st.gap_finish &&
                       a.OH == 1 && a.OW == 1 && a.R == is.h && a.S == is.w && a.pad == 0 && is.n <= 32 && !st.scalar && a.C == is.c &&
                       ((long long)a.R * a.S * a.C) % 64 == 0 && (long long)a.R * a.S * a.C >= 512 && (long long)a.R * a.S * a.C < (1ll << 30) &&
                       iv.sN % p.ce == 0 && iv.sN >= (long long)a.R * a.S * a.C && (a.R * a.S == 1 || (iv.sP == a.C && iv.sN == (long long)a.R * a.S * a.C));
        {
          const int src_node = nd.in[0] - 1;
          pack_shuffle_groups = !is_fc && src_node >= 0 && nodes[src_node].kind == XENOS_OP_SHUFFLE && fold_shuffle[src_node] ? desc(nodes[src_node]).groups : 0;
        }
        pack_dense(st, go, is_fc ? is.c : is.c, a.C, a.R, a.S, K);
        pack_shuffle_groups = 0;
        push_affine(af, (K + 127) / 128 * 128, &st.scale_off, &st.shift_off);
        if (st.scalar) {
          std::vector<int32_t> tab((size_t)2 * a.Kred_pad);
          for (int kk = 0; kk < a.Kred_pad; ++kk) {
            if (kk < a.Kred) {
              const int c = kk % a.C, rs = kk / a.C, s = rs % a.S, r = rs / a.S;
              tab[2 * kk] = (int32_t)(r * a.in_sH + s * a.in_sW + c * iv.sK);
              tab[2 * kk + 1] = (r << 16) | s;
            } else {
              tab[2 * kk] = 0;
              tab[2 * kk + 1] = (0x4000 << 16);   // row far outside any map: contributes zero
            }
          }
          st.ktab_off = (long long)wpush(tab.data(), tab.size() * 4);
        }
        finish(last, cur, true);
        const View& ov = p.views[st.v_out];
        a.out_sN = ov.sN; a.out_sP = ov.sP; a.out_sK = ov.sK; a.out_f32 = ov.f32;
        // 16-byte channel-group accesses need unit channel stride, the compute type and aligned slices
        a.vec_out = ov.sK == 1 && (!ov.f32 || p.dt == DT_F32) && ov.esz == p.esz && K % p.ce == 0 && ov.off % p.ce == 0 &&
                    ov.sP % p.ce == 0 && ov.sN % p.ce == 0;
        if (a.ileave && !a.vec_out) return fail(XENOS_EUNSUPPORTED, "%s: shuffled concat buffer is not aligned", st.name.c_str());
        if (has_res) {
          const View& rv = p.views[st.v_in2];
          a.vec_res = K % p.ce == 0 && rv.off % p.ce == 0 && rv.sP % p.ce == 0 && rv.sN % p.ce == 0;
        }
        if (dw_panel_fits && a.mode == M_FLAT && (a.vec_out || st.gap_finish)) {
          // depthwise panel on chip: as many input channels as fit the unit's private memory beside the weight stages
          const int bke = kRowBytes / p.esz, cpad = (a.C + bke - 1) / bke * bke;
          int cp = cpad;
          while (cp > bke && dwpw_lds_bytes(cp, p.esz) > std::min<size_t>(p.hw.lds_bytes_per_cu, 160 * 1024)) cp -= bke;
          if (dwpw_lds_bytes(cp, p.esz) <= std::min<size_t>(p.hw.lds_bytes_per_cu, 160 * 1024)) a.dw_panel = cp;
        }
        xenos_status rc = split_conv(st);
        if (rc != XENOS_OK) return rc;
        if (a.dw_panel > 0) st.lds = dwpw_lds_bytes(a.dw_panel, p.esz);
        st.flops = 2.0 * a.N * a.OH * a.OW * (double)K * a.R * a.S * is.c + (from_dw ? pro.flops : 0.0) + (from_pair ? ppro.flops : 0.0);
        if (from_dw) st.bytes_w += pro.bytes_w;
        if (from_pair) st.bytes_w += ppro.bytes_w;
        st.bytes_in = view_bytes(st.v_in); st.bytes_out = view_bytes(st.v_out);
        if (has_res || a.ileave) st.bytes_res = view_bytes(st.v_in2);

        // Parameter split beyond K (Section 4.2.2: C, R, S splits need an extra reduction): when the outC x H/W
        // partition leaves most compute units idle and the reduction is long, split it across workgroups too.
        // Shares are summed in index order by a second pass, so the result does not depend on timing.
        // the convolution step hands a.ksplit shares of raw sums [share][pixel][a.part_ld] to a summing pass, which
        // applies the chain's epilogue (scale, shift, shortcut, ReLU, global average) and stores the chain's output
        auto emit_with_summing_pass = [&]() -> xenos_status {
          const int ks = a.ksplit;
          View pv;
          pv.esz = 4; pv.f32 = 1; pv.s = Shape{1, 1, 1, 1};
          const long long pbytes = (long long)ks * a.M_total * a.part_ld * 4;
          pv.buf = new_buffer(pbytes, 0);
          p.views.push_back(pv);
          const int v_part = (int)p.views.size() - 1;
          Step fin;
          fin.kind = S_SPLITK; fin.name = st.name + ".sum";
          fin.ops = st.ops;                                      // the summing pass completes the same chain
          fin.v_in = v_part; fin.v_in2 = st.v_in2; fin.v_out = st.v_out;
          fin.scale_off = st.scale_off; fin.shift_off = st.shift_off;
          SplitKArgs& f = fin.splitk;
          f.ksplit = ks; f.part_ld = a.part_ld; f.M = a.M_total; f.K = K; f.OHW = a.OH * a.OW;
          f.res_sN = a.res_sN; f.res_sP = a.res_sP;
          f.out_sN = a.out_sN; f.out_sP = a.out_sP; f.out_sK = a.out_sK; f.relu = a.relu; f.out_f32 = a.out_f32;
          f.gap = st.gap_finish;
          fin.bytes_in = pbytes; fin.bytes_res = st.bytes_res; fin.bytes_out = st.bytes_out;
          st.v_out = v_part; st.v_in2 = -1; a.has_res = 0;
          // (the halo kernel finds a pixel's row of the partial sums through the output strides)
          if (st.cfg == kHaloCfg) { a.out_sN = (long long)a.OH * a.OW * a.part_ld; a.out_sP = a.part_ld; a.out_sK = 1; }
          st.bytes_out = pbytes; st.bytes_res = 0;
          const int sidx = (int)p.steps.size();
          node_step[i] = sidx + 1;
          for (int ab : absorbed) node_step[ab] = sidx + 1;
          node_final[last] = 1;
          add_step(st);
          add_step(fin);
          return XENOS_OK;
        };
        if (hsplit.ks >= 2) {
          const ConvArgs& t = hsplit.tile;
          a.th = t.th; a.tw = t.tw; a.tiles_y = t.tiles_y; a.tiles_x = t.tiles_x; a.tiles_m = t.tiles_m;
          a.halo_plin = 0; a.halo_bn = t.halo_bn; a.tiles_n = t.tiles_n; a.ntiles = t.ntiles;
          st.cfg = kHaloCfg; st.lds = conv_lds_bytes(kHaloCfg, M_FLAT);
          st.cands.clear();                                        // the plan's structure depends on this split
          a.ksplit = hsplit.ks; a.steps_per_split = a.C / (kRowBytes / p.esz) / hsplit.ks;
          a.part_ld = a.tiles_n * a.halo_bn;
          set_grid(a, kHaloCfg);
          return emit_with_summing_pass();
        }
        const int nsteps = a.Kred_pad / (kRowBytes / p.esz);
        if (st.fc_stream || (p.opts.split && !a.ileave && st.cfg < kHaloCfg && a.mode == M_FLAT && (!from_dw || (st.gap_finish && a.dw_panel > 0)) &&
            (st.gap_finish || (a.ntiles * 2 <= p.hw.num_cu && nsteps >= 16)))) {
          int ks = std::min({(2 * p.hw.num_cu + a.ntiles - 1) / a.ntiles, nsteps / 2, 32});
          if (st.gap_finish) ks = std::max(ks, 1);
          if (from_dw) ks = 1;                                     // the depthwise-panel kernel hands over one share
          const int fc_tiles = (K + kFcChannels - 1) / kFcChannels;
          // (two workgroups per unit, each with at least 4 steps = 32 KB of weights to stream)
          if (st.fc_stream) ks = std::max(1, std::min((kFcWgPerCu * std::max(1, p.hw.num_cu) + fc_tiles - 1) / fc_tiles, nsteps / 4));
          if (st.fc_stream && nsteps <= kFcDirectSteps && !has_res) {
            // short reduction: one share per channel tile, epilogue in the streaming kernel, no summing pass (one launch
            // fewer where launches are what a pass costs: the classifier of a batch-1 network)
            st.cands.clear();
            st.cfg = kFcCfg; st.lds = 0;
            a.ksplit = 0; a.steps_per_split = nsteps;
            // (a workgroup per 32 channels, the steps dealt to its four wavefronts)
            a.tiles_m = 1; a.tiles_n = fc_tiles; a.ntiles = fc_tiles; a.xcd_m = 1; a.grid = (K + 31) / 32;
          } else
          if (st.fc_stream || ks >= 4 || st.gap_finish) {
            const int spk = (nsteps + ks - 1) / ks;
            ks = (nsteps + spk - 1) / spk;
            st.cands.clear();                                      // the plan's structure now depends on this tile shape
            a.ksplit = ks; a.steps_per_split = spk;
            if (st.fc_stream) {
              st.cfg = kFcCfg; st.lds = 0;
              a.tiles_m = 1; a.tiles_n = fc_tiles; a.ntiles = fc_tiles; a.xcd_m = 1;
              a.part_ld = fc_tiles * kFcChannels;
              a.grid = fc_tiles * ks;
            } else {
              a.part_ld = a.tiles_n * kTileCfgs[st.cfg].bn;
              set_grid(a, st.cfg);
            }
            return emit_with_summing_pass();
          }
        }
      }
      const int sidx = (int)p.steps.size();
      node_step[i] = sidx;
      for (int a : absorbed) node_step[a] = sidx;
      node_final[last] = 1;
      add_step(st);
      return XENOS_OK;
    }
  }

  // ---- pointwise chain -> depthwise chain as ONE step (pwdw_kernel); the checks are pwdw_consumer's ---------------
  xenos_status plan_pwdw(int i, const ChainWalk& w1, int dn) {
    const Node& nd = nodes[i];
    const GOp& go = g.ops[nd.src];
    const Node& dnode = nodes[dn];
    const xenos_op_desc& dd = desc(dnode);
    const Shape is = tshape[nd.in[0]], os = tshape[dn + 1];
    const int K = desc(nd).out_c;
    const ChainWalk w2 = walk_chain(dn);
    Step st;
    st.kind = S_CONV;
    st.name = std::string("op") + std::to_string(nd.src);
    st.ops.push_back(nd.src);
    for (int a : w1.absorbed) st.ops.push_back(nodes[a].src);
    st.ops.push_back(dnode.src);
    for (int a : w2.absorbed) st.ops.push_back(nodes[a].src);
    st.v_in = tview[nd.in[0]];
    const View& iv = p.views[st.v_in];
    ConvArgs& a = st.conv;
    a.N = is.n; a.C = std::max(is.c, iv.cphys); a.H = is.h; a.W = is.w; a.K = K;   // (padding channels multiply zero weights)
    a.R = 1; a.S = 1; a.stride = 1; a.pad = 0; a.OH = os.h; a.OW = os.w; a.PH = os.h; a.PW = os.w;
    a.in_sN = iv.sN; a.in_sH = iv.sP * is.w; a.in_sW = iv.sP;
    a.relu = w1.relu; a.mode = M_FLAT; a.pool = POOL_NONE;
    a.pwdw = 1; a.dw_k = 3; a.dw_stride = dd.stride_h; a.dw_pad = 1; a.dw_relu = w2.relu; a.dw_H = is.h; a.dw_W = is.w;
    a.M_total = a.N * a.OH * a.OW;
    pack_dense(st, go, is.c, a.C, 1, 1, K);
    push_affine(w1.af, (K + 127) / 128 * 128, &st.scale_off, &st.shift_off);
    st.dw_w_off = pack_depthwise(g.ops[dnode.src], K, 9);
    push_affine(w2.af, (K + 63) / 64 * 64, &st.dw_scale_off, &st.dw_shift_off);
    st.v_out = out_view_for(w2.cur, true);
    const View& ov = p.views[st.v_out];
    a.out_sN = ov.sN; a.out_sP = ov.sP; a.out_sK = ov.sK; a.out_f32 = ov.f32;
    a.vec_out = ov.sK == 1 && !ov.f32 && ov.esz == p.esz && ov.off % p.ce == 0 && ov.sP % p.ce == 0 && ov.sN % p.ce == 0;
    if (!a.vec_out) return fail(XENOS_EUNSUPPORTED, "%s: output of the pointwise -> depthwise chain is not aligned", st.name.c_str());
    if (!choose_pwdw_tile(a)) return fail(XENOS_EUNSUPPORTED, "%s: no tile of the pointwise -> depthwise kernel fits", st.name.c_str());
    a.tiles_m = a.N * a.tiles_y * a.tiles_x;
    a.tiles_n = (K + kPwDwChannels - 1) / kPwDwChannels;
    a.ntiles = a.tiles_m * a.tiles_n;
    a.xcd_m = 8;
    a.grid = p.opts.split ? std::max(1, std::min(a.ntiles, 4 * std::max(1, p.hw.num_cu))) : 1;
    st.cfg = kPwDwCfg;
    st.lds = pwdw_lds_bytes(a.th, a.tw, a.dw_stride, p.esz);
    st.flops = 2.0 * is.n * is.h * is.w * (double)K * is.c + 2.0 * os.n * os.h * os.w * (double)K * 9;
    st.bytes_w += (long long)9 * K * p.esz;
    st.bytes_in = view_bytes(st.v_in); st.bytes_out = view_bytes(st.v_out);
    const int sidx = (int)p.steps.size();
    node_step[i] = sidx; node_step[dn] = sidx;
    for (int ab : w1.absorbed) node_step[ab] = sidx;
    for (int ab : w2.absorbed) node_step[ab] = sidx;
    node_final[w2.last] = 1;
    add_step(st);
    return XENOS_OK;
  }

  // ---- stand-alone operators: whatever the link pass did not absorb into a convolution chain ---------------------
  xenos_status plan_standalone(int i) {
    const Node& nd = nodes[i];
    const xenos_op_desc& d = desc(nd);
    const GOp& go = g.ops[nd.src];
    const Shape is = tshape[nd.in[0]];
    Step st;
    st.name = std::string("op") + std::to_string(nd.src);
    st.ops.push_back(nd.src);
    if (nd.kind == XENOS_OP_CONCAT && free_concat[i]) {
      out_view_for(i + 1, false);          // the buffer exists; producers write their slices into it
      node_step[i] = std::max(0, (int)p.steps.size() - 1);
      node_final[i] = 1;
      return XENOS_OK;
    }
    if (nd.kind == XENOS_OP_CONCAT && ileave[i]) {
      // interleaved concat (a channel shuffle linked into it): parts stored by their chains are in place already,
      // the others are copied to their channel positions
      const int ov = out_view_for(i + 1, false);
      if (!p.views[ov].internal_nhwc() || p.views[ov].f32) return fail(XENOS_EUNSUPPORTED, "concat output must be internal");
      for (size_t j = 0; j < nd.in.size(); ++j) {
        if (placed.count(nd.in[j]) || fin_concat[i]) continue;
        Step cs;
        cs.kind = S_ELT; cs.name = st.name + ".part" + std::to_string(j);
        cs.ops.push_back(nd.src);
        xenos_status rc = need_internal_input(nd.in[j], cs.name.c_str(), &cs.v_in);
        if (rc != XENOS_OK) return rc;
        View sl = p.views[ov];
        sl.s = tshape[nd.in[j]]; sl.off += (long long)j; sl.sK = ileave[i];
        p.views.push_back(sl);
        cs.v_out = tag((int)p.views.size() - 1, nd.in[j]);
        fill_elt(cs, ELT_COPY, 0);
        add_step(cs);
      }
      node_step[i] = std::max(0, (int)p.steps.size() - 1);
      node_final[i] = 1;
      return XENOS_OK;
    }
    if (nd.kind == XENOS_OP_SHUFFLE && (alias_shuffle[i] || fold_shuffle[i])) {
      if (tview[nd.in[0]] < 0) return fail(XENOS_EINVAL, "%s: input not materialised", st.name.c_str());
      tview[i + 1] = tview[nd.in[0]];
      node_step[i] = std::max(0, (int)p.steps.size() - 1);
      node_final[i] = 1;
      ++p.n_linked_shuffles;
      return XENOS_OK;
    }
    if (nd.kind == XENOS_OP_SHUFFLE) {
      // stand-alone shuffle: one strided copy per group (group j of the input goes to channels j, j + g, ...)
      const int g = d.groups, m = is.c / g;
      int vin;
      xenos_status rc = need_internal_input(nd.in[0], st.name.c_str(), &vin);
      if (rc != XENOS_OK) return rc;
      const int ov = out_view_for(i + 1, false);
      if (!p.views[ov].internal_nhwc() || p.views[ov].f32) return fail(XENOS_EUNSUPPORTED, "%s: output must be internal", st.name.c_str());
      const bool whole = g == 1 || m == 1;                         // one group, or one channel per group: a plain copy
      for (int j = 0; j < (whole ? 1 : g); ++j) {
        Step cs;
        cs.kind = S_ELT; cs.name = st.name + ".group" + std::to_string(j);
        cs.ops.push_back(nd.src);
        View a = p.views[vin], o = p.views[ov];
        if (!whole) {
          a.s.c = m; a.off += (long long)j * m * a.sK;
          o.s.c = m; o.off += (long long)j * o.sK; o.sK *= g;
        }
        p.views.push_back(a); cs.v_in = (int)p.views.size() - 1;
        p.views.push_back(o); cs.v_out = (int)p.views.size() - 1;
        if (!whole) {   // group j of the input; its channels land at j, j + g, ... of the output
          p.views[cs.v_in].gc0 += j * m * p.views[cs.v_in].gcs;
          tag(cs.v_out, i + 1, j, g);
        }
        fill_elt(cs, ELT_COPY, 0);
        add_step(cs);
      }
      node_step[i] = (int)p.steps.size() - 1;
      node_final[i] = 1;
      return XENOS_OK;
    }
    if (nd.kind == XENOS_OP_SLICE) {
      // a channel range of a tensor is a view of it; only a slice that is the graph output is copied
      int vin;
      xenos_status rc = need_internal_input(nd.in[0], st.name.c_str(), &vin);
      if (rc != XENOS_OK) return rc;
      View sl = p.views[vin];
      sl.s = tshape[i + 1]; sl.off += (long long)d.c_begin * sl.sK;
      if (sl.cphys) sl.cphys = 0;
      p.views.push_back(sl);
      const int sv = tag((int)p.views.size() - 1, i + 1);
      // (a range that does not start and end on a 16-byte channel group is copied too: the vector loaders of its
      // consumers need aligned groups)
      if (i + 1 == out_tid || placed.count(i + 1) || sl.off % p.ce != 0 || sl.s.c % p.ce != 0) {
        st.kind = S_ELT;
        st.v_in = sv;
        st.v_out = out_view_for(i + 1, false);
        if (p.views[st.v_out].f32) return fail(XENOS_EUNSUPPORTED, "%s: output must be internal", st.name.c_str());
        fill_elt(st, ELT_COPY, 0);
        add_step(st);
        node_step[i] = (int)p.steps.size() - 1;
      } else {
        tview[i + 1] = sv;
        node_step[i] = std::max(0, (int)p.steps.size() - 1);
      }
      node_final[i] = 1;
      return XENOS_OK;
    }
    if (nd.kind == XENOS_OP_CONCAT) {
      const int ov = out_view_for(i + 1, false);
      if (!p.views[ov].internal_nhwc() || p.views[ov].f32) return fail(XENOS_EUNSUPPORTED, "concat output must be internal");
      int off = 0;
      for (size_t j = 0; j < nd.in.size(); ++j) {
        Step cs;
        cs.kind = S_ELT; cs.name = st.name + ".part" + std::to_string(j);
        cs.ops.push_back(nd.src);
        xenos_status rc = need_internal_input(nd.in[j], cs.name.c_str(), &cs.v_in);
        if (rc != XENOS_OK) return rc;
        View sl = p.views[ov];
        sl.s = tshape[nd.in[j]]; sl.off += off;
        p.views.push_back(sl);
        cs.v_out = tag((int)p.views.size() - 1, nd.in[j]);
        fill_elt(cs, ELT_COPY, 0);
        add_step(cs);
        off += tshape[nd.in[j]].c;
      }
      node_step[i] = (int)p.steps.size() - 1;
      node_final[i] = 1;
      return XENOS_OK;
    }

    xenos_status rc = need_internal_input(nd.in[0], st.name.c_str(), &st.v_in);
    if (rc != XENOS_OK) return rc;
    if (nd.kind == XENOS_OP_ADD) {
      rc = need_internal_input(nd.in[1], st.name.c_str(), &st.v_in2);
      if (rc != XENOS_OK) return rc;
    }
    st.v_out = out_view_for(i + 1, false);
    if (!p.views[st.v_out].internal_nhwc() || p.views[st.v_out].f32)
      return fail(XENOS_EUNSUPPORTED, "%s: output must be internal", st.name.c_str());
    switch (nd.kind) {
      case XENOS_OP_BIAS:
      case XENOS_OP_BN: {
        Affine af;
        af.scale.assign(is.c, 1.0);
        af.shift.assign(is.c, 0.0);
        if (nd.kind == XENOS_OP_BIAS) fold_bias(af, go.bias); else fold_bn(af, go);
        st.kind = S_ELT;
        push_affine(af, is.c, &st.scale_off, &st.shift_off);
        fill_elt(st, ELT_AFFINE, 0);
        break;
      }
      case XENOS_OP_RELU: st.kind = S_ELT; fill_elt(st, ELT_RELU, 0); break;
      case XENOS_OP_ADD: st.kind = S_ELT; fill_elt(st, ELT_ADD, 0); break;
      case XENOS_OP_MAXPOOL:
      case XENOS_OP_AVGPOOL:
      case XENOS_OP_GLOBAL_AVGPOOL: {
        st.kind = S_POOL;
        PoolArgs& a = st.pool;
        const View& iv = p.views[st.v_in];
        const View& ov = p.views[st.v_out];
        const Shape os = tshape[i + 1];
        a.N = is.n; a.C = is.c; a.H = is.h; a.W = is.w; a.OH = os.h; a.OW = os.w;
        a.k = d.kh; a.s = d.stride_h; a.p = d.pad_h; a.cip = d.count_include_pad;
        a.kind = nd.kind == XENOS_OP_MAXPOOL ? POOL_MAX : nd.kind == XENOS_OP_AVGPOOL ? POOL_AVG : POOL_GAP;
        a.in_sN = iv.sN; a.in_sP = iv.sP; a.out_sN = ov.sN; a.out_sP = ov.sP;
        st.bytes_in = view_bytes(st.v_in); st.bytes_out = view_bytes(st.v_out);
        break;
      }
      default: return fail(XENOS_EUNSUPPORTED, "operator kind %d", nd.kind);
    }
    node_step[i] = (int)p.steps.size();
    node_final[i] = 1;
    add_step(st);
    return XENOS_OK;
  }

  void fill_elt(Step& st, int op, int relu) {
    EltArgs& e = st.elt;
    const View& a = p.views[st.v_in];
    const View& o = p.views[st.v_out];
    e.op = op; e.relu = relu; e.C = a.s.c;
    e.pixels = (long long)a.s.n * a.s.h * a.s.w;
    e.a_sP = a.sP; e.out_sP = o.sP; e.a_sK = a.sK; e.out_sK = o.sK;
    if (st.v_in2 >= 0) e.b_sP = p.views[st.v_in2].sP;
    st.bytes_in = view_bytes(st.v_in) + (st.v_in2 >= 0 ? view_bytes(st.v_in2) : 0);
    st.bytes_out = view_bytes(st.v_out);
  }

  // ---- workspace allocation with liveness (first fit) -------------------------------------------
  void allocate() {
    struct Blk { size_t off, size; };
    std::vector<Blk> free_list;
    size_t top = 0;
    const int ns = (int)p.steps.size();
    std::vector<std::vector<int>> born(ns + 1), dies(ns + 1);
    for (int b = 0; b < (int)p.bufs.size(); ++b) {
      Buffer& bf = p.bufs[b];
      if (bf.ext || bf.last < 0) continue;
      born[bf.first].push_back(b);
      dies[bf.last].push_back(b);
    }
    for (int s = 0; s < ns; ++s) {
      for (int b : born[s]) {
        const size_t need = align_up((size_t)p.bufs[b].bytes + 64, 256);   // slack: vector loads never cross the end
        size_t got = (size_t)-1;
        for (size_t k = 0; k < free_list.size(); ++k)
          if (free_list[k].size >= need) {
            got = free_list[k].off;
            free_list[k].off += need; free_list[k].size -= need;
            if (free_list[k].size == 0) free_list.erase(free_list.begin() + k);
            break;
          }
        if (got == (size_t)-1) { got = top; top += need; }
        p.bufs[b].offset = got;
        p.bufs[b].bytes = (long long)need;
      }
      for (int b : dies[s]) {
        Blk nb{p.bufs[b].offset, (size_t)p.bufs[b].bytes};
        free_list.push_back(nb);
        // coalesce
        std::sort(free_list.begin(), free_list.end(), [](const Blk& x, const Blk& y) { return x.off < y.off; });
        for (size_t k = 0; k + 1 < free_list.size();)
          if (free_list[k].off + free_list[k].size == free_list[k + 1].off) {
            free_list[k].size += free_list[k + 1].size;
            free_list.erase(free_list.begin() + k + 1);
          } else ++k;
      }
    }
    p.workspace_bytes = std::max<size_t>(top, 256);
  }

  void write_json() { write_plan_json(p); }
};

// The plan's metadata as JSON (Section 4.1 "metadata"): chains, tiles, layouts, algorithmic work.
void write_plan_json(xenos_plan& p) {
  std::string& j = p.json;
  char buf[1024];
  double tf = 0; long long tb = 0;
  for (const Step& s : p.steps) { tf += s.flops; tb += s.bytes_in + s.bytes_w + s.bytes_out + s.bytes_res; }
  snprintf(buf, sizeof buf, "{\"link\":%d,\"split\":%d,\"compute\":\"%s\",\"num_cu\":%d,\"n_chains\":%d,\"flops\":%.0f,\"hbm_bytes\":%lld,"
           "\"linked_shuffles\":%d,\"weight_bytes\":%zu,\"workspace_bytes\":%zu,\"chains\":[",
           p.opts.link, p.opts.split, p.dt == DT_BF16 ? "bf16" : "f32", p.hw.num_cu, (int)p.steps.size(), tf, tb,
           p.n_linked_shuffles, p.wimage.size(), p.workspace_bytes);
  j = buf;
  for (size_t i = 0; i < p.steps.size(); ++i) {
    const Step& s = p.steps[i];
    std::string ops;
    for (size_t k = 0; k < s.ops.size(); ++k) ops += (k ? "," : "") + std::to_string(s.ops[k]);
    snprintf(buf, sizeof buf, "%s{\"i\":%d,\"name\":\"%s\",\"kind\":\"%s\",\"ops\":[%s],\"flops\":%.0f,\"bytes_in\":%lld,\"bytes_w\":%lld,"
             "\"bytes_out\":%lld,\"bytes_res\":%lld",
             i ? "," : "", (int)i, s.name.c_str(), kStepNames[s.kind], ops.c_str(), s.flops, s.bytes_in, s.bytes_w, s.bytes_out, s.bytes_res);
    j += buf;
    if (s.kind == S_CONV) {
      const ConvArgs& c = s.conv;
      const TileCfg halo_tc{kHaloRows, c.halo_bn, 64, c.halo_bn / 2};
      const TileCfg stem_tc{32, c.K, 32, c.K};
      const TileCfg pair_tc{kPairRows, kPairChannels, 64, kPairChannels / 2};
      const TileCfg fc_tc{32, kFcChannels, 32, 32};
      const TileCfg stem_lds_tc{kStemLdsTh * kStemLdsTw, c.K, 32, c.K};
      const TileCfg pwdw_tc{64, kPwDwChannels, 32, 32};
      const TileCfg& tc = s.cfg == kPwDwCfg || s.cfg == kFireCfg ? pwdw_tc : s.cfg == kHaloCfg ? halo_tc : s.cfg == kStemCfg ? stem_tc : s.cfg == kStemLdsCfg ? stem_lds_tc : s.cfg == kPairCfg ? pair_tc : s.cfg == kFcCfg ? fc_tc : kTileCfgs[s.cfg];
      snprintf(buf, sizeof buf, ",\"mode\":\"%s\",\"loader\":\"%s\",\"N\":%d,\"C\":%d,\"H\":%d,\"W\":%d,\"K\":%d,\"R\":%d,\"S\":%d,\"stride\":%d,"
               "\"pad\":%d,\"OH\":%d,\"OW\":%d,\"PH\":%d,\"PW\":%d,\"pool\":%d,\"relu\":%d,\"res\":%d,\"bm\":%d,\"bn\":%d,\"tiles_m\":%d,"
               "\"tiles_n\":%d,\"grid\":%d,\"lds\":%zu,\"pph\":%d,\"ppw\":%d,\"patch_h\":%d,\"patch_w\":%d,\"out_c_off\":%lld,\"out_sP\":%lld,\"halo\":%d,\"th\":%d,\"tw\":%d,\"dw_linked\":%d,\"ksplit\":%d,\"candidates\":%d,\"tuned\":%d,\"plin\":%d,\"shuffle_store\":%d",
               kModeNames[c.mode], s.stem ? "stem" : c.pair ? "pair" : c.pwdw ? "pwdw" : c.fire ? "fire" : s.fc_stream ? "stream" : s.scalar ? "scalar" : "vector", c.N, c.C, c.H, c.W, c.K, c.R, c.S, c.stride, c.pad, c.OH, c.OW,
               c.PH, c.PW, c.pool, c.relu, c.has_res, tc.bm, tc.bn, c.tiles_m, c.tiles_n, c.grid, s.lds, c.pph, c.ppw, c.patch_h,
               c.patch_w, p.views[s.v_out].off, c.out_sP, s.cfg == kHaloCfg ? 1 : 0, c.th, c.tw, s.dw_w_off >= 0 ? 1 : 0, c.ksplit > 1 ? c.ksplit : 1, (int)s.cands.size(), s.tuned, s.cfg == kHaloCfg ? c.halo_plin : 0, c.ileave);
      j += buf;
    }
    // where the chain's tensors lie (byte offset into the workspace / the caller's input or output buffer, element
    // strides) and which graph tensor each one is
    auto view_json = [&](const char* key, int v) {
      if (v < 0) return;
      const View& vw = p.views[v];
      const Buffer& bf = p.bufs[vw.buf];
      snprintf(buf, sizeof buf, ",\"%s\":{\"mem\":\"%s\",\"byte_off\":%lld,\"sN\":%lld,\"sP\":%lld,\"sK\":%lld,\"esz\":%d,\"f32\":%d,"
               "\"n\":%d,\"c\":%d,\"h\":%d,\"w\":%d,\"cphys\":%d,\"tensor\":%d,\"c0\":%d,\"cs\":%d}",
               key, bf.ext == 1 ? "input" : bf.ext == 2 ? "output" : "workspace", (long long)(bf.ext ? 0 : bf.offset) + vw.off * vw.esz,
               vw.sN, vw.sP, vw.sK, vw.esz, vw.f32, vw.s.n, vw.s.c, vw.s.h, vw.s.w, vw.cphys, vw.gt, vw.gc0, vw.gcs);
      j += buf;
    };
    view_json("in", s.v_in);
    view_json("in2", s.v_in2);
    view_json("out", s.v_out);
    view_json("out2", s.v_out2);
    j += "}";
  }
  j += "]}";
}

// ---------------------------------------------------------------------------------------------
// Runtime
// ---------------------------------------------------------------------------------------------
// `ws`: the workspace the intermediate tensors live in (the bound one, or the library's static one)
struct Mem { const void* d_in; void* d_out; const void* ws; };

const unsigned char* view_ptr(const xenos_plan& p, int v, const Mem& m) {
  const View& vw = p.views[v];
  const Buffer& b = p.bufs[vw.buf];
  const unsigned char* base = b.ext == 1 ? (const unsigned char*)m.d_in
                              : b.ext == 2 ? (const unsigned char*)m.d_out
                                           : (const unsigned char*)m.ws + b.offset;
  return base + vw.off * vw.esz;
}

xenos_status launch_step(xenos_plan& p, const Step& s, const void* d_in_, void* d_out_, void* stream, const void* ws = nullptr) {
  const Mem mem{d_in_, d_out_, ws ? ws : p.d_workspace};
  const unsigned char* wb = (const unsigned char*)p.d_weights;
  int rc = 0;
  switch (s.kind) {
    case S_CONV: {
      ConvArgs a = s.conv;
      a.in = view_ptr(p, s.v_in, mem);
      a.out = (void*)view_ptr(p, s.v_out, mem);
      a.res = s.v_in2 >= 0 ? view_ptr(p, s.v_in2, mem) : nullptr;
      a.zeros = wb + p.zero_off;
      a.w = wb + s.w_off;
      a.scale = (const float*)(wb + s.scale_off);
      a.shift = (const float*)(wb + s.shift_off);
      a.ktab = s.ktab_off >= 0 ? (const int32_t*)(wb + s.ktab_off) : nullptr;
      a.part = a.ksplit >= 1 ? (float*)a.out : nullptr;
      a.dw_w = s.dw_w_off >= 0 ? (const void*)(wb + s.dw_w_off) : nullptr;
      a.dw_scale = s.dw_scale_off >= 0 ? (const float*)(wb + s.dw_scale_off) : nullptr;
      a.dw_shift = s.dw_shift_off >= 0 ? (const float*)(wb + s.dw_shift_off) : nullptr;
      if (a.fire) {
        for (int e = 0; e < 2; ++e) {
          const bool has = a.fire_E[e] > 0;
          a.fire_w[e] = has ? wb + s.fire_w_off[e] : nullptr;
          a.fire_scale[e] = has ? (const float*)(wb + s.fire_scale_off[e]) : nullptr;
          a.fire_shift[e] = has ? (const float*)(wb + s.fire_shift_off[e]) : nullptr;
        }
        a.fire_out[0] = a.fire_E[0] > 0 ? a.out : nullptr;
        a.fire_out[1] = a.fire_E[1] > 0 ? (void*)view_ptr(p, s.v_out2, mem) : nullptr;
      }
      rc = launch_conv(a, p.dt, s.cfg, s.scalar, stream);
      break;
    }
    case S_DW: {
      DwArgs a = s.dw;
      a.in = view_ptr(p, s.v_in, mem);
      a.out = (void*)view_ptr(p, s.v_out, mem);
      a.w = wb + s.w_off;
      a.scale = (const float*)(wb + s.scale_off);
      a.shift = (const float*)(wb + s.shift_off);
      rc = launch_dw(a, p.dt, stream);
      break;
    }
    case S_ELT: {
      EltArgs a = s.elt;
      a.a = view_ptr(p, s.v_in, mem);
      a.b = s.v_in2 >= 0 ? view_ptr(p, s.v_in2, mem) : nullptr;
      a.out = (void*)view_ptr(p, s.v_out, mem);
      a.scale = s.scale_off >= 0 ? (const float*)(wb + s.scale_off) : nullptr;
      a.shift = s.shift_off >= 0 ? (const float*)(wb + s.shift_off) : nullptr;
      rc = launch_elt(a, p.dt, stream);
      break;
    }
    case S_POOL: {
      PoolArgs a = s.pool;
      a.in = view_ptr(p, s.v_in, mem);
      a.out = (void*)view_ptr(p, s.v_out, mem);
      rc = launch_pool(a, p.dt, stream);
      break;
    }
    case S_SPLITK: {
      SplitKArgs a = s.splitk;
      a.part = (const float*)view_ptr(p, s.v_in, mem);
      a.res = s.v_in2 >= 0 ? view_ptr(p, s.v_in2, mem) : nullptr;
      a.out = (void*)view_ptr(p, s.v_out, mem);
      a.scale = (const float*)(wb + s.scale_off);
      a.shift = (const float*)(wb + s.shift_off);
      rc = launch_splitk_finish(a, p.dt, stream);
      break;
    }
    case S_CVT: {
      CvtArgs a = s.cvt;
      a.in = view_ptr(p, s.v_in, mem);
      a.out = (void*)view_ptr(p, s.v_out, mem);
      rc = launch_cvt(a, p.dt, stream);
      break;
    }
  }
  if (rc != 0) return fail(XENOS_EDEVICE, "launch of chain %s failed: %s", s.name.c_str(), hipGetErrorString((hipError_t)rc));
  return XENOS_OK;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// Workspace of xenos_run_static: a file-scope device array instead of caller memory.  Every GPU the library runs on
// holds its own copy for the life of the process.  In host code the array's name is only a handle for
// hipGetSymbolAddress; its device address is looked up once per device and kept.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[XENOS_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the current device (nullptr + message on failure)
void* static_workspace() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(XENOS_EDEVICE, "xenos_run_static: no current device (%s)", hipGetErrorString(e));
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      fail(XENOS_EDEVICE, "xenos_run_static: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------------
extern "C" {

const char* xenos_last_error(void) { return g_err.c_str(); }

xenos_status xenos_graph_create(const xenos_tensor_desc* input, const xenos_op_desc* ops, int n_ops,
                                int output_tensor_id, const xenos_tensor_desc* output, xenos_graph** out) {
  if (!input || !ops || !out || n_ops <= 0) return fail(XENOS_EINVAL, "xenos_graph_create: NULL argument or no operators");
  if (input->n <= 0 || input->c <= 0 || input->h <= 0 || input->w <= 0) return fail(XENOS_ESHAPE, "input shape must be positive");
  if (output_tensor_id <= 0 || output_tensor_id > n_ops) return fail(XENOS_EINVAL, "output tensor id %d out of range", output_tensor_id);
  xenos_graph* g = new (std::nothrow) xenos_graph;
  if (!g) return fail(XENOS_ENOMEM, "out of host memory");
  g->in = *input;
  g->shapes.push_back(Shape{input->n, input->c, input->h, input->w});
  g->output_id = output_tensor_id;
  xenos_status rc = XENOS_OK;
  try {
    for (int i = 0; i < n_ops && rc == XENOS_OK; ++i) {
      const xenos_op_desc& d = ops[i];
      GOp o;
      o.d = d;
      o.d.weight = o.d.bias = o.d.gamma = o.d.beta = o.d.mean = o.d.var = nullptr;
      const int want_in = d.kind == XENOS_OP_ADD ? 2 : d.kind == XENOS_OP_CONCAT ? d.n_inputs : 1;
      if (d.n_inputs != want_in || d.n_inputs < 1 || d.n_inputs > 4 || (d.kind == XENOS_OP_CONCAT && d.n_inputs < 2)) {
        rc = fail(XENOS_EINVAL, "op %d: wrong number of inputs (%d)", i, d.n_inputs);
        break;
      }
      for (int j = 0; j < d.n_inputs; ++j)
        if (d.inputs[j] < 0 || d.inputs[j] > i) { rc = fail(XENOS_EINVAL, "op %d: input %d is not an earlier tensor", i, d.inputs[j]); break; }
      if (rc != XENOS_OK) break;
      const Shape s = g->shapes[d.inputs[0]];
      Shape os = s;
      auto need = [&](const float* ptr, size_t n, std::vector<float>& dst, const char* what, bool required) {
        if (!ptr) {
          if (required) rc = fail(XENOS_EINVAL, "op %d: missing %s", i, what);
          return;
        }
        dst.assign(ptr, ptr + n);
      };
      switch (d.kind) {
        case XENOS_OP_CONV: {
          if (d.kh <= 0 || d.kw <= 0 || d.stride_h <= 0 || d.out_c <= 0 || d.groups <= 0 || d.pad_h < 0)
            { rc = fail(XENOS_EINVAL, "op %d: bad conv attributes", i); break; }
          if (d.stride_h != d.stride_w || d.pad_h != d.pad_w) { rc = fail(XENOS_EUNSUPPORTED, "op %d: stride/pad must be equal in h and w", i); break; }
          if (s.c % d.groups || d.out_c % d.groups) { rc = fail(XENOS_ESHAPE, "op %d: channels not divisible by groups", i); break; }
          if (s.h + 2 * d.pad_h < d.kh || s.w + 2 * d.pad_w < d.kw) { rc = fail(XENOS_ESHAPE, "op %d: kernel larger than padded map", i); break; }
          if (d.kh >= 0x4000 || d.kw >= 0x4000) { rc = fail(XENOS_EUNSUPPORTED, "op %d: kernel too large", i); break; }
          os = Shape{s.n, d.out_c, (s.h + 2 * d.pad_h - d.kh) / d.stride_h + 1, (s.w + 2 * d.pad_w - d.kw) / d.stride_w + 1};
          need(d.weight, (size_t)d.out_c * (s.c / d.groups) * d.kh * d.kw, o.weight, "weight", true);
          need(d.bias, d.out_c, o.bias, "bias", false);
          break;
        }
        case XENOS_OP_FC:
          if (d.out_c <= 0) { rc = fail(XENOS_EINVAL, "op %d: bad fc attributes", i); break; }
          os = Shape{s.n, d.out_c, 1, 1};
          need(d.weight, (size_t)d.out_c * s.c * s.h * s.w, o.weight, "weight", true);
          need(d.bias, d.out_c, o.bias, "bias", false);
          break;
        case XENOS_OP_MATMUL:
          if (d.out_c <= 0) { rc = fail(XENOS_EINVAL, "op %d: bad matmul attributes", i); break; }
          if (s.h != 1 || s.w != 1) { rc = fail(XENOS_ESHAPE, "op %d: matmul takes an M x K x 1 x 1 tensor (rows x columns), got %dx%dx%dx%d", i, s.n, s.c, s.h, s.w); break; }
          os = Shape{s.n, d.out_c, 1, 1};
          need(d.weight, (size_t)d.out_c * s.c, o.weight, "weight", true);
          need(d.bias, d.out_c, o.bias, "bias", false);
          break;
        case XENOS_OP_BIAS: need(d.bias, s.c, o.bias, "bias", true); break;
        case XENOS_OP_BN:
          need(d.gamma, s.c, o.gamma, "gamma", true);
          need(d.beta, s.c, o.beta, "beta", true);
          need(d.mean, s.c, o.mean, "mean", true);
          need(d.var, s.c, o.var, "var", true);
          if (rc == XENOS_OK)
            for (int k = 0; k < s.c; ++k)
              if (!(o.var[k] + d.eps > 0.f)) { rc = fail(XENOS_EINVAL, "op %d: var + eps must be positive", i); break; }
          break;
        case XENOS_OP_RELU: break;
        case XENOS_OP_MAXPOOL:
        case XENOS_OP_AVGPOOL:
          if (d.kh <= 0 || d.kh != d.kw || d.stride_h <= 0 || d.stride_h != d.stride_w || d.pad_h != d.pad_w || d.pad_h < 0 || 2 * d.pad_h > d.kh)
            { rc = fail(XENOS_EUNSUPPORTED, "op %d: pooling needs a square window, equal strides and pad <= k/2", i); break; }
          if (s.h + 2 * d.pad_h < d.kh || s.w + 2 * d.pad_w < d.kw) { rc = fail(XENOS_ESHAPE, "op %d: pooling window larger than map", i); break; }
          os = Shape{s.n, s.c, pool_out(s.h, d.kh, d.stride_h, d.pad_h, d.ceil_mode), pool_out(s.w, d.kw, d.stride_w, d.pad_w, d.ceil_mode)};
          break;
        case XENOS_OP_GLOBAL_AVGPOOL: os = Shape{s.n, s.c, 1, 1}; break;
        case XENOS_OP_ADD: {
          const Shape b = g->shapes[d.inputs[1]];
          if (b.n != s.n || b.c != s.c || b.h != s.h || b.w != s.w) rc = fail(XENOS_ESHAPE, "op %d: add operands differ in shape", i);
          break;
        }
        case XENOS_OP_CONCAT: {
          int ct = 0;
          for (int j = 0; j < d.n_inputs; ++j) {
            const Shape b = g->shapes[d.inputs[j]];
            if (b.n != s.n || b.h != s.h || b.w != s.w) rc = fail(XENOS_ESHAPE, "op %d: concat operands differ in N/H/W", i);
            ct += b.c;
          }
          os.c = ct;
          break;
        }
        case XENOS_OP_SLICE:
          if (d.c_begin < 0 || d.out_c <= 0 || (long long)d.c_begin + d.out_c > s.c)
            { rc = fail(XENOS_ESHAPE, "op %d: slice [%d, %d + %d) outside the %d channels of its input", i, d.c_begin, d.c_begin, d.out_c, s.c); break; }
          os.c = d.out_c;
          break;
        case XENOS_OP_SHUFFLE:
          if (d.groups <= 0 || s.c % d.groups) { rc = fail(XENOS_ESHAPE, "op %d: %d channels not divisible by %d shuffle groups", i, s.c, d.groups); break; }
          break;
        default: rc = fail(XENOS_EINVAL, "op %d: unknown kind %d", i, (int)d.kind);
      }
      if (rc != XENOS_OK) break;
      if (os.h <= 0 || os.w <= 0) { rc = fail(XENOS_ESHAPE, "op %d: empty output", i); break; }
      g->shapes.push_back(os);
      g->ops.push_back(std::move(o));
    }
  } catch (const std::bad_alloc&) {
    rc = fail(XENOS_ENOMEM, "out of host memory");
  }
  if (rc != XENOS_OK) { delete g; return rc; }
  const Shape os = g->shapes[output_tensor_id];
  xenos_tensor_desc od{os.n, os.c, os.h, os.w, XENOS_F32, XENOS_NCHW};
  if (output) {
    if ((output->n && output->n != os.n) || (output->c && output->c != os.c) || (output->h && output->h != os.h) || (output->w && output->w != os.w)) {
      delete g;
      return fail(XENOS_ESHAPE, "output descriptor %dx%dx%dx%d does not match inferred %dx%dx%dx%d", output->n, output->c, output->h, output->w, os.n, os.c, os.h, os.w);
    }
    od.dtype = output->dtype; od.layout = output->layout;
  }
  g->out = od;
  *out = g;
  return XENOS_OK;
}

xenos_status xenos_plan_link_split(const xenos_graph* graph, const xenos_hw_info* hw, const xenos_plan_opts* opts, xenos_plan** out) {
  if (!graph || !hw || !opts || !out || graph->magic != MAGIC_GRAPH) return fail(XENOS_EINVAL, "xenos_plan_link_split: bad argument");
  if (opts->link < 0 || opts->link > 3 || opts->tile < 0 || opts->tile > kNumTileCfgs + 6 || (opts->compute != XENOS_F32 && opts->compute != XENOS_BF16))
    return fail(XENOS_EINVAL, "xenos_plan_link_split: option out of range");
  if (hw->num_cu <= 0 || hw->lds_bytes_per_cu == 0) return fail(XENOS_EINVAL, "xenos_plan_link_split: hardware description is empty");
  if ((graph->in.dtype == XENOS_BF16 || graph->out.dtype == XENOS_BF16) && opts->compute != XENOS_BF16)
    return fail(XENOS_EUNSUPPORTED, "bf16 graph input/output needs the bf16 compute type");
  xenos_plan* p = new (std::nothrow) xenos_plan;
  if (!p) return fail(XENOS_ENOMEM, "out of host memory");
  p->opts = *opts; p->hw = *hw; p->in = graph->in; p->out = graph->out;
  xenos_status rc;
  try {
    Planner pl(*graph, *p);
    rc = pl.run();
  } catch (const std::bad_alloc&) {
    rc = fail(XENOS_ENOMEM, "out of host memory");
  }
  if (rc != XENOS_OK) { delete p; return rc; }
  *out = p;
  return XENOS_OK;
}

xenos_status xenos_plan_query(const xenos_plan* plan, size_t* weight_bytes, size_t* workspace_bytes, xenos_tensor_desc* out_desc,
                              char* json, size_t json_cap, size_t* json_len) {
  if (!plan || plan->magic != MAGIC_PLAN) return fail(XENOS_EINVAL, "xenos_plan_query: bad plan");
  if (weight_bytes) *weight_bytes = std::max<size_t>(plan->wimage.size(), 256);
  if (workspace_bytes) *workspace_bytes = plan->workspace_bytes;
  if (out_desc) *out_desc = plan->out;
  if (json_len) *json_len = plan->json.size() + 1;
  if (json && json_cap) {
    const size_t n = std::min(json_cap - 1, plan->json.size());
    memcpy(json, plan->json.data(), n);
    json[n] = 0;
  }
  return XENOS_OK;
}

xenos_status xenos_plan_bind(xenos_plan* plan, void* d_weights, void* d_workspace, void* hip_stream) {
  // (d_workspace may be NULL: the plan can then run through xenos_run_static only)
  if (!plan || plan->magic != MAGIC_PLAN || !d_weights) return fail(XENOS_EINVAL, "xenos_plan_bind: bad argument");
  if (((uintptr_t)d_weights | (uintptr_t)d_workspace) & 255) return fail(XENOS_EINVAL, "xenos_plan_bind: buffers must be 256-byte aligned");
  hipStream_t st = (hipStream_t)hip_stream;
  if (!plan->wimage.empty()) {
    hipError_t e = hipMemcpyAsync(d_weights, plan->wimage.data(), plan->wimage.size(), hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return fail(XENOS_EDEVICE, "weight upload failed: %s", hipGetErrorString(e));
  }
  hipError_t e = hipStreamSynchronize(st);
  if (e != hipSuccess) return fail(XENOS_EDEVICE, "stream synchronise failed: %s", hipGetErrorString(e));
  plan->d_weights = d_weights;
  plan->d_workspace = d_workspace;
  plan->bound = true;
  return XENOS_OK;
}

xenos_status xenos_run(xenos_plan* plan, const void* d_input, void* d_output, void* hip_stream) {
  if (!plan || plan->magic != MAGIC_PLAN || !d_input || !d_output) return fail(XENOS_EINVAL, "xenos_run: bad argument");
  if (!plan->bound) return fail(XENOS_EINVAL, "xenos_run: plan is not bound (call xenos_plan_bind)");
  if (!plan->d_workspace) return fail(XENOS_EINVAL, "xenos_run: the plan was bound without a workspace (xenos_run_static only)");
  for (const Step& s : plan->steps) {
    xenos_status rc = launch_step(*plan, s, d_input, d_output, hip_stream);
    if (rc != XENOS_OK) return rc;
  }
  return XENOS_OK;
}

xenos_status xenos_run_with(xenos_plan* plan, const void* d_input, void* d_output, void* d_workspace, void* hip_stream) {
  if (!plan || plan->magic != MAGIC_PLAN || !d_input || !d_output || !d_workspace) return fail(XENOS_EINVAL, "xenos_run_with: bad argument");
  if (!plan->bound) return fail(XENOS_EINVAL, "xenos_run_with: plan is not bound (call xenos_plan_bind)");
  if ((uintptr_t)d_workspace & 255) return fail(XENOS_EINVAL, "xenos_run_with: the workspace must be 256-byte aligned");
  // The pass reads the plan (host) and the weight image (device) and writes only d_workspace and d_output, so passes
  // with different workspaces and outputs do not touch each other's memory.
  for (const Step& s : plan->steps) {
    xenos_status rc = launch_step(*plan, s, d_input, d_output, hip_stream, d_workspace);
    if (rc != XENOS_OK) return rc;
  }
  return XENOS_OK;
}

xenos_status xenos_run_static(xenos_plan* plan, const void* d_input, void* d_output, void* hip_stream) {
  if (!plan || plan->magic != MAGIC_PLAN || !d_input || !d_output) return fail(XENOS_EINVAL, "xenos_run_static: bad argument");
  if (!plan->bound) return fail(XENOS_EINVAL, "xenos_run_static: plan is not bound (call xenos_plan_bind)");
  if (plan->workspace_bytes > (size_t)XENOS_STATIC_WORKSPACE_BYTES)
    return fail(XENOS_EUNSUPPORTED, "xenos_run_static: the plan needs %zu bytes of workspace, the static workspace holds %zu",
                plan->workspace_bytes, (size_t)XENOS_STATIC_WORKSPACE_BYTES);
  void* ws = static_workspace();
  if (!ws) return XENOS_EDEVICE;
  // No chain reads a workspace byte that an earlier chain of the same pass (or the weight image) has not written, so
  // nothing is cleared: what the previous call left behind is overwritten before it is read.
  for (const Step& s : plan->steps) {
    xenos_status rc = launch_step(*plan, s, d_input, d_output, hip_stream, ws);
    if (rc != XENOS_OK) return rc;
  }
  return XENOS_OK;
}

xenos_status xenos_run_graph(xenos_plan* plan, const void* d_input, void* d_output, void* hip_stream) {
  if (!plan || plan->magic != MAGIC_PLAN || !d_input || !d_output) return fail(XENOS_EINVAL, "xenos_run_graph: bad argument");
  if (!plan->bound || !plan->d_workspace) return fail(XENOS_EINVAL, "xenos_run_graph: plan is not bound to a workspace (call xenos_plan_bind)");
  auto key = std::make_pair(d_input, d_output);
  auto it = plan->graphs.find(key);
  if (it == plan->graphs.end()) {
    // capture the kernel sequence (kernel nodes only) on a private stream of default priority
    if (!plan->capture_stream) {
      hipError_t e = hipStreamCreateWithFlags(&plan->capture_stream, hipStreamNonBlocking);
      if (e != hipSuccess) return fail(XENOS_EDEVICE, "stream create failed: %s", hipGetErrorString(e));
    }
    hipError_t e = hipStreamBeginCapture(plan->capture_stream, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) return fail(XENOS_EDEVICE, "graph capture failed to start: %s", hipGetErrorString(e));
    xenos_status rc = XENOS_OK;
    for (const Step& s : plan->steps) {
      rc = launch_step(*plan, s, d_input, d_output, plan->capture_stream);
      if (rc != XENOS_OK) break;
    }
    hipGraph_t graph = nullptr;
    e = hipStreamEndCapture(plan->capture_stream, &graph);
    if (rc != XENOS_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    if (e != hipSuccess || !graph) return fail(XENOS_EDEVICE, "graph capture failed: %s", hipGetErrorString(e));
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return fail(XENOS_EDEVICE, "graph instantiate failed: %s", hipGetErrorString(e));
    it = plan->graphs.emplace(key, exec).first;
  }
  hipError_t e = hipGraphLaunch(it->second, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(XENOS_EDEVICE, "graph launch failed: %s", hipGetErrorString(e));
  return XENOS_OK;
}

xenos_status xenos_plan_tune(xenos_plan* plan, const void* d_input, void* d_output, void* hip_stream, int reps, int* n_changed) {
  if (!plan || plan->magic != MAGIC_PLAN || !d_input || !d_output || reps < 1) return fail(XENOS_EINVAL, "xenos_plan_tune: bad argument");
  if (!plan->bound || !plan->d_workspace) return fail(XENOS_EINVAL, "xenos_plan_tune: plan is not bound to a workspace (call xenos_plan_bind)");
  hipStream_t st = (hipStream_t)hip_stream;
  // one full pass first: every buffer then holds finite values of the real shapes (workspace blocks are reused along the
  // pass, so a chain is not guaranteed to find its own input there; run times do not depend on the values)
  for (const Step& s : plan->steps) {
    xenos_status rc = launch_step(*plan, s, d_input, d_output, hip_stream);
    if (rc != XENOS_OK) return rc;
  }
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
    if (e0) (void)hipEventDestroy(e0);
    return fail(XENOS_EDEVICE, "xenos_plan_tune: event create failed");
  }
  int changed = 0;
  xenos_status rc = XENOS_OK;
  for (Step& s : plan->steps) {
    if (s.kind != S_CONV || s.cands.size() < 2) continue;
    int best = -1, incumbent = -1;                                // incumbent: the cost model's choice among the candidates
    float best_ms = 0.f, incumbent_ms = 0.f;
    for (size_t ci = 0; ci < s.cands.size() && rc == XENOS_OK; ++ci) {
      Step trial = s;
      trial.cfg = s.cands[ci].cfg; trial.conv = s.cands[ci].a; trial.lds = s.cands[ci].lds;
      if (launch_step(*plan, trial, d_input, d_output, hip_stream) != XENOS_OK) continue;   // warm-up; a candidate that cannot launch is skipped
      if (hipEventRecord(e0, st) != hipSuccess) { rc = fail(XENOS_EDEVICE, "xenos_plan_tune: event record failed"); break; }
      for (int r = 0; r < reps; ++r) (void)launch_step(*plan, trial, d_input, d_output, hip_stream);
      float ms = 0.f;
      if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
        rc = fail(XENOS_EDEVICE, "xenos_plan_tune: timing failed");
        break;
      }
      if (best < 0 || ms < best_ms) { best = (int)ci; best_ms = ms; }
      const Step::Cand& cc = s.cands[ci];
      if (cc.cfg == s.cfg && cc.a.tiles_m == s.conv.tiles_m && cc.a.tiles_n == s.conv.tiles_n && cc.a.halo_bn == s.conv.halo_bn &&
          cc.a.halo_plin == s.conv.halo_plin) { incumbent = (int)ci; incumbent_ms = ms; }
    }
    if (rc != XENOS_OK) break;
    // a few short trials time a chain to 2-3 %: the cost model's choice is given up only for a clear win
    if (best >= 0 && incumbent >= 0 && best != incumbent && best_ms > 0.96f * incumbent_ms) { best = incumbent; best_ms = incumbent_ms; }
    if (best >= 0) {
      const Step::Cand& c = s.cands[best];
      const bool same = c.cfg == s.cfg && c.a.tiles_m == s.conv.tiles_m && c.a.tiles_n == s.conv.tiles_n && c.a.halo_bn == s.conv.halo_bn && c.a.halo_plin == s.conv.halo_plin;
      if (!same) ++changed;
      s.cfg = c.cfg; s.conv = c.a; s.lds = c.lds; s.tuned = 1;
      // the last trial may not have been the winner: leave the winner's output in the workspace for the next chain
      if (launch_step(*plan, s, d_input, d_output, hip_stream) != XENOS_OK) { rc = fail(XENOS_EDEVICE, "xenos_plan_tune: launch failed"); break; }
    }
  }
  // a full pass with the chosen partitions leaves the output valid
  if (rc == XENOS_OK)
    for (const Step& s : plan->steps) {
      rc = launch_step(*plan, s, d_input, d_output, hip_stream);
      if (rc != XENOS_OK) break;
    }
  (void)hipStreamSynchronize(st);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  // graphs captured before the choice are stale
  for (auto& kv : plan->graphs) (void)hipGraphExecDestroy(kv.second);
  plan->graphs.clear();
  write_plan_json(*plan);
  if (n_changed) *n_changed = changed;
  return rc;
}

xenos_status xenos_run_chain(xenos_plan* plan, int chain, const void* d_input, void* d_output, void* hip_stream) {
  if (!plan || plan->magic != MAGIC_PLAN || !d_input || !d_output) return fail(XENOS_EINVAL, "xenos_run_chain: bad argument");
  if (!plan->bound || !plan->d_workspace) return fail(XENOS_EINVAL, "xenos_run_chain: plan is not bound to a workspace");
  if (chain < 0 || chain >= (int)plan->steps.size()) return fail(XENOS_EINVAL, "xenos_run_chain: chain %d out of range", chain);
  return launch_step(*plan, plan->steps[chain], d_input, d_output, hip_stream);
}

xenos_status xenos_probe_mfma(const xenos_hw_info* hw, void* d_out, size_t out_bytes, int iters, int data, void* hip_stream, double* flops) {
  if (!hw || hw->num_cu <= 0 || !d_out || iters < 1 || data < 0 || data > 2) return fail(XENOS_EINVAL, "xenos_probe_mfma: bad argument");
  if (out_bytes < probe_out_bytes(hw->num_cu)) return fail(XENOS_EINVAL, "xenos_probe_mfma: d_out must hold %zu bytes", probe_out_bytes(hw->num_cu));
  const int rc = launch_probe_mfma(d_out, hw->num_cu, iters, data, hip_stream, flops);
  if (rc != 0) return fail(XENOS_EDEVICE, "xenos_probe_mfma: launch failed: %s", hipGetErrorString((hipError_t)rc));
  return XENOS_OK;
}

xenos_status xenos_probe_read(const xenos_hw_info* hw, const void* d_in, size_t bytes, void* d_out, size_t out_bytes, void* hip_stream) {
  if (!hw || hw->num_cu <= 0 || !d_in || !d_out || bytes < 16 || (bytes & 15) || ((uintptr_t)d_in & 15))
    return fail(XENOS_EINVAL, "xenos_probe_read: bad argument (bytes and d_in must be multiples of 16)");
  if (out_bytes < probe_out_bytes(hw->num_cu)) return fail(XENOS_EINVAL, "xenos_probe_read: d_out must hold %zu bytes", probe_out_bytes(hw->num_cu));
  const int rc = launch_probe_read(d_in, bytes, d_out, hw->num_cu, hip_stream);
  if (rc != 0) return fail(XENOS_EDEVICE, "xenos_probe_read: launch failed: %s", hipGetErrorString((hipError_t)rc));
  return XENOS_OK;
}

void xenos_destroy(void* h) {
  if (!h) return;
  const uint32_t magic = *(const uint32_t*)h;
  if (magic == MAGIC_GRAPH) { ((xenos_graph*)h)->magic = 0; delete (xenos_graph*)h; }
  else if (magic == MAGIC_PLAN) { ((xenos_plan*)h)->magic = 0; delete (xenos_plan*)h; }
}

}  // extern "C"
