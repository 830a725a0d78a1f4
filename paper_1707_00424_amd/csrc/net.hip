// Replica-batched network executor.  A network is a static list of ops over tensors that live in
// the caller's workspace; every op is one (or a few) grouped launches covering all replicas.
// The backward pass walks the list in reverse with hand-written gradient routing (which tensor
// receives which gradient, written or accumulated) fixed at plan time.
#include <stdlib.h>

#include <algorithm>

#include "net.h"

#include "igemm.h"
#include "nn.h"

namespace {

enum OpType { OP_CONV = 0, OP_POOL = 1, OP_GAP = 2, OP_BNRELU = 3, OP_DROP = 4 };

struct Tensor {
  int H = 0, W = 0, C = 0;
  bool f32 = false;       // fp32 storage regardless of the activation dtype (logits)
  bool external = false;  // the caller's image buffer (fp32 mode): no workspace slot
  int64_t off = -1;       // byte offset in the workspace
  int64_t goff = -1;      // byte offset of its gradient (activation dtype), -1 = none
};

struct Op {
  int type = 0;
  int in = -1, out = -1;
  // conv / fc
  int wseg = -1, bseg = -1;
  int Hin = 0, Win = 0, Cin = 0, Cout = 0, R = 1, stride = 1, pad = 0, Ho = 0, Wo = 0;
  bool relu = false;
  int resid = -1;          // tensor added to the conv output before the ReLU
  bool need_dx = false;
  bool mask_in = false;    // the input is a ReLU output: its gradient is masked by (in > 0)
  bool dx_accumulate = false;
  int dy = -1;             // tensor whose gradient is this op's output gradient (default: out)
  // A shortcut convolution is a branch beside the block's chain of convolutions: it runs on the second stream
  // (forward), and its input gradient, which needs only the block output's gradient, is written there as soon
  // as that gradient is final; the block's first convolution, whose input is the same tensor, then
  // accumulates its own input gradient onto it.
  bool branch = false;     // this op is such a shortcut
  int join = -1;           // index of the shortcut op whose output this op reads (resid) and whose backward it starts
  int dx_after = -1;       // index of the shortcut op whose input gradient this op's accumulates onto
  int64_t wt_off = -1;     // transposed weights (bytes)
  int64_t col_off = -1;    // per-tap products of the two-pass backward-data (bytes), -1 = direct kernel
  bool win = false;        // backward-data through per-tap products held in LDS, one image per workgroup
  // pool
  bool pool_relu_mask = false;
  // bn
  int gseg = -1, betaseg = -1;
  int64_t saved_off = -1, sums_off = -1, run_off = 0;  // run_off in floats inside a replica's BN row
  int bn_add = -1;         // tensor whose gradient is added to this op's input gradient
  int stat_src = -1;       // the convolution that writes this op's input, if its epilogue can take the column sums
  // conv / fc: the classifier's last layer.  In training its forward pass, the loss and its input gradient run as
  // one kernel (launch_fc_head) in place of three on the chain; its weight and bias gradients stay as they are.
  bool head = false;
  // dropout
  int site = 0;            // index of the dropout site in execution order (part of the mask's key)
  bool drop_relu = false;  // the input is a ReLU output whose backward mask this op applies
};

}  // namespace

struct Net {
  parle_config cfg;
  Arch arch;
  std::vector<Segment> segs;
  int64_t n_pad = 0;
  int n = 0, B = 0, dtype = 0, esize = 4;
  std::vector<Tensor> tensors;
  std::vector<Op> ops;
  int t_images = -1, t_logits = -1;
  int64_t ws_bytes = 0;
  int64_t off_colpartial = 0, off_wpartial = 0, off_rowcopy = 0, wpartial_bytes = 0, wpartial_main_bytes = 0;
  // Weight and bias gradients are leaves of the backward pass: they run on a second stream beside the
  // chain of input gradients (own column-partial scratch; the weight partials are used there only).
  int64_t off_colpartial_side = 0;
  // Bias gradients (two small kernels per layer) on a third stream: they would otherwise sit in the second
  // stream's queue in front of every weight gradient.
  hipStream_t side2 = nullptr;
  hipEvent_t side2_done = nullptr;
  // All of a network's bias gradients or none: networks of small layers (LeNet, the MLP) lose more to the extra
  // events than the stream hides (+4 %), and a mix of both placements measured worst of all.
  bool bias_stream = false;
  bool bias_in_wgrad = true;  // PARLE_BIAS_IN_WGRAD=0: every bias gradient by its own column-sum kernels
  // bf16 networks: the first layer gathers the caller's fp32 images itself, rounding as it gathers, where its
  // kernels can (the small-window ones); otherwise a bf16 copy is made first.  PARLE_IMAGES_DIRECT=0: always copy.
  int images_reader = -1;  // the one convolution that reads the images, or -1
  // Wavefronts a weight-gradient launch of the nine-tap kernel puts in flight.  Where batch-norm passes share
  // the chain of input gradients, that chain is the longer one and the leaves have slack: they take half the
  // chip's SIMDs and leave the rest to the chain (WRN-16-4 -3 %); without batch-norm the leaves are the longer
  // side and take all of them (All-CNN-C: +3.7 % with half).
  int leaf_waves = 0;
  // A layer without input gradient (the first one) is the last the backward pass reaches: nothing follows it on
  // the first stream, so its leaves run there, beside whatever the second stream still has queued (own scratch).
  int64_t off_wpartial_main = 0;
  bool overlap = true;
  hipStream_t side = nullptr;
  std::vector<hipEvent_t> dy_ready;  // one per op: its output gradient is final
  // per op, used by shortcut ops only: input ready (forward fork), output ready (forward join), input gradient
  // ready (backward join)
  std::vector<hipEvent_t> br_fork, br_out, br_dx;
  hipEvent_t side_done = nullptr;
  hipEvent_t step_begin = nullptr, wt_ready = nullptr;  // the weight transposes of a step run beside its forward pass
  ~Net() {
    if (step_begin) (void)hipEventDestroy(step_begin);
    if (wt_ready) (void)hipEventDestroy(wt_ready);
    for (const std::vector<hipEvent_t> *v : {&dy_ready, &br_fork, &br_out, &br_dx})
      for (hipEvent_t e : *v)
        if (e) (void)hipEventDestroy(e);
    if (side_done) (void)hipEventDestroy(side_done);
    if (side2_done) (void)hipEventDestroy(side2_done);
    if (side) (void)hipStreamDestroy(side);
    if (side2) (void)hipStreamDestroy(side2);
  }
  int64_t bn_floats = 0;
  int max_bn_c = 0;
  int head_op = -1;          // index of the op with `head` set, -1 = the network ends otherwise
  int64_t off_loss_img = 0;  // [n][B] per-image losses
  std::vector<TransposeTable> transposes;  // weights that backward-data reads transposed, in launch-sized groups

  int64_t alloc(int64_t bytes) {
    const int64_t o = ws_bytes;
    ws_bytes += (bytes + 255) / 256 * 256;
    return o;
  }
  int add_tensor(int H, int W, int C, bool f32 = false, bool external = false) {
    Tensor t;
    t.H = H, t.W = W, t.C = C, t.f32 = f32, t.external = external;
    if (!external) t.off = alloc((int64_t)n * B * H * W * C * (f32 ? 4 : esize));
    tensors.push_back(t);
    return (int)tensors.size() - 1;
  }
  void want_grad(int t) {
    if (tensors[t].goff < 0) tensors[t].goff = alloc((int64_t)n * B * tensors[t].H * tensors[t].W * tensors[t].C * esize);
  }
  int64_t rs(int t) const { return (int64_t)B * tensors[t].H * tensors[t].W * tensors[t].C; }

  // conv on tensor `in` seen as [B, Hin, Win, Cin]; returns the op index
  int add_conv(int in, int Hin, int Win, int Cin, const std::string &name, int Cout, int R, int stride, int pad,
               bool bias, bool relu, bool out_f32 = false) {
    Op op;
    op.type = OP_CONV;
    op.in = in;
    op.Hin = Hin, op.Win = Win, op.Cin = Cin, op.Cout = Cout, op.R = R, op.stride = stride, op.pad = pad;
    op.Ho = (Hin + 2 * pad - R) / stride + 1;
    op.Wo = (Win + 2 * pad - R) / stride + 1;
    op.relu = relu;
    op.wseg = find_segment(segs, name + ".w");
    op.bseg = bias ? find_segment(segs, name + ".b") : -1;
    op.out = add_tensor(op.Ho, op.Wo, Cout, out_f32);
    op.dy = op.out;
    ops.push_back(op);
    return (int)ops.size() - 1;
  }
  int add_bn(int in, const std::string &name) {
    Op op;
    op.type = OP_BNRELU;
    op.in = in;
    const Tensor t = tensors[in];  // copy: add_tensor may reallocate the vector
    op.out = add_tensor(t.H, t.W, t.C);
    op.gseg = find_segment(segs, name + ".g");
    op.betaseg = find_segment(segs, name + ".b");
    op.saved_off = alloc((int64_t)n * 2 * t.C * 4);
    op.sums_off = alloc((int64_t)n * 2 * t.C * 4);
    op.run_off = bn_floats;
    bn_floats += 2 * t.C;
    if (t.C > max_bn_c) max_bn_c = t.C;
    ops.push_back(op);
    return (int)ops.size() - 1;
  }
  int n_drop_sites = 0;
  // dropout on tensor `in` (no-op when the rate is zero): returns the tensor the next layer reads
  int add_drop(int in, bool relu_input) {
    if (!(cfg.dropout > 0.f)) return in;
    Op op;
    op.type = OP_DROP;
    op.in = in;
    const Tensor t = tensors[in];
    op.out = add_tensor(t.H, t.W, t.C);
    op.site = n_drop_sites++;
    op.drop_relu = relu_input;
    ops.push_back(op);
    return op.out;
  }
};

namespace {

bool build_plan(Net &N, std::string &err) {
  const Arch &a = N.arch;
  const bool bf = N.dtype == 1;
  // the images: fp32 mode reads the caller's buffer directly, bf16 mode converts into a slot
  N.t_images = N.add_tensor(a.H, a.W, a.C, false, !bf);
  const int img = N.t_images;
  switch (a.model) {
    case PARLE_MODEL_MLP: {
      const int d = a.H * a.W * a.C;
      const int f1 = N.add_conv(img, 1, 1, d, "fc1", a.a0, 1, 1, 0, true, true);
      const int f2 = N.add_conv(N.ops[f1].out, 1, 1, a.a0, "fc2", a.classes, 1, 1, 0, true, false, true);
      N.ops[f2].need_dx = true, N.ops[f2].mask_in = true;
      N.t_logits = N.ops[f2].out;
      break;
    }
    case PARLE_MODEL_LENET: {
      const int k = a.a2;
      const bool bn = a.bn != 0, drop = N.cfg.dropout > 0.f;
      // conv (+ ReLU in its epilogue, or batch-norm + ReLU as an op of its own), pooling, dropout
      const int c1 = N.add_conv(img, a.H, a.W, a.C, "conv1", a.a0, k, 1, 0, true, !bn);
      int h1 = N.ops[c1].out;
      if (bn) h1 = N.ops[N.add_bn(h1, "bn1")].out;
      Op p1;
      p1.type = OP_POOL, p1.in = h1, p1.pool_relu_mask = !bn;
      p1.out = N.add_tensor(N.ops[c1].Ho / 2, N.ops[c1].Wo / 2, a.a0);
      N.ops.push_back(p1);
      const Tensor tp1 = N.tensors[p1.out];
      const int d1 = N.add_drop(p1.out, false);
      const int c2 = N.add_conv(d1, tp1.H, tp1.W, a.a0, "conv2", a.a1, k, 1, 0, true, !bn);
      N.ops[c2].need_dx = true;
      int h2 = N.ops[c2].out;
      if (bn) h2 = N.ops[N.add_bn(h2, "bn2")].out;
      Op p2;
      p2.type = OP_POOL, p2.in = h2, p2.pool_relu_mask = !bn;
      p2.out = N.add_tensor(N.ops[c2].Ho / 2, N.ops[c2].Wo / 2, a.a1);
      N.ops.push_back(p2);
      const Tensor tp2 = N.tensors[p2.out];
      const int d2 = N.add_drop(p2.out, false);
      const int f1 = N.add_conv(d2, 1, 1, tp2.H * tp2.W * tp2.C, "fc1", a.a3, 1, 1, 0, true, !bn);
      N.ops[f1].need_dx = true;
      int h3 = N.ops[f1].out;
      if (bn) h3 = N.ops[N.add_bn(h3, "bn3")].out;
      // the ReLU mask of fc1's output is applied by whoever writes its gradient: fc2's backward-data, or the
      // dropout in between; after batch-norm the batch-norm backward applies it itself
      const int d3 = N.add_drop(h3, !bn);
      const int f2 = N.add_conv(d3, 1, 1, a.a3, "fc2", a.classes, 1, 1, 0, true, false, true);
      N.ops[f2].need_dx = true, N.ops[f2].mask_in = !bn && !drop;
      N.t_logits = N.ops[f2].out;
      break;
    }
    case PARLE_MODEL_ALLCNN_C: {
      const int ca = a.a0, cb = a.a1;
      const int cout[9] = {ca, ca, ca, cb, cb, cb, cb, cb, a.classes};
      const int ks[9] = {3, 3, 3, 3, 3, 3, 3, 1, 1};
      const int st[9] = {1, 1, 2, 1, 1, 2, 1, 1, 1};
      int cur = img, H = a.H, W = a.W, C = a.C;
      for (int i = 0; i < 9; ++i) {
        const int c = N.add_conv(cur, H, W, C, "conv" + std::to_string(i + 1), cout[i], ks[i], st[i], ks[i] == 3 ? 1 : 0,
                                 true, i < 8);
        // the gradient of a ReLU output is masked by its consumer: the next conv, or the dropout in between
        const bool after_drop = N.cfg.dropout > 0.f && i > 0 && st[i - 1] == 2;
        if (i > 0) N.ops[c].need_dx = true, N.ops[c].mask_in = !after_drop;
        cur = N.ops[c].out, H = N.ops[c].Ho, W = N.ops[c].Wo, C = cout[i];
        if (st[i] == 2) cur = N.add_drop(cur, true);
      }
      Op g;
      g.type = OP_GAP, g.in = cur;
      g.out = N.add_tensor(1, 1, C, true);
      N.ops.push_back(g);
      N.t_logits = g.out;
      break;
    }
    case PARLE_MODEL_WRN: {
      const int c0 = N.add_conv(img, a.H, a.W, a.C, "conv1", a.a0, 3, 1, 1, false, false);
      int h = N.ops[c0].out, H = N.ops[c0].Ho, W = N.ops[c0].Wo;
      for (const WrnBlock &b : wrn_block_list(a)) {
        const int bn1 = N.add_bn(h, b.name + ".bn1");
        const int o = N.ops[bn1].out;
        int s = -1, sc = -1;
        if (b.has_sc) {
          sc = N.add_conv(o, H, W, b.cin, b.name + ".sc", b.cout, 1, b.stride, 0, false, false);
          N.ops[sc].need_dx = true, N.ops[sc].branch = true;
          s = N.ops[sc].out;
        } else {
          N.ops[bn1].bn_add = -2;  // resolved below to the block output
        }
        const int cv1 = N.add_conv(o, H, W, b.cin, b.name + ".conv1", b.cout, 3, b.stride, 1, false, false);
        N.ops[cv1].need_dx = true;
        if (b.has_sc) N.ops[cv1].dx_accumulate = true, N.ops[cv1].dx_after = sc;
        const int bn2 = N.add_bn(N.ops[cv1].out, b.name + ".bn2");
        const int cv1_ho = N.ops[cv1].Ho, cv1_wo = N.ops[cv1].Wo;
        const int mid = N.add_drop(N.ops[bn2].out, false);
        const int cv2 = N.add_conv(mid, cv1_ho, cv1_wo, b.cout, b.name + ".conv2", b.cout, 3, 1, 1, false, false);
        N.ops[cv2].need_dx = true;
        N.ops[cv2].resid = b.has_sc ? s : h;
        const int v = N.ops[cv2].out;
        if (b.has_sc) {
          // the shortcut conv's output gradient is the block output's gradient
          N.ops[sc].dy = v, N.ops[cv2].join = sc;
        } else {
          N.ops[bn1].bn_add = v;
        }
        h = v, H = cv1_ho, W = cv1_wo;
      }
      const int bno = N.add_bn(h, "bn_out");
      Op g;
      g.type = OP_GAP, g.in = N.ops[bno].out;
      g.out = N.add_tensor(1, 1, N.tensors[h].C, false);
      N.ops.push_back(g);
      const int fc = N.add_conv(g.out, 1, 1, N.tensors[h].C, "fc", a.classes, 1, 1, 0, true, false, true);
      N.ops[fc].need_dx = true;
      N.t_logits = N.ops[fc].out;
      break;
    }
    default:
      err = "model has no network";
      return false;
  }
  {
    static const bool fused_head = [] {
      const char *e = getenv("PARLE_FUSED_HEAD");
      return !(e && atoi(e) == 0);
    }();
    Op &last = N.ops.back();
    if (fused_head && last.type == OP_CONV && last.out == N.t_logits && N.tensors[last.out].f32 && last.R == 1 &&
        last.Hin == 1 && last.Win == 1 && last.stride == 1 && last.pad == 0 && last.need_dx && last.resid < 0 &&
        !last.relu && fc_head_applicable(last.Cout, last.Cin) && last.Cin <= 256) {
      // up to 256 features: MLP (128) -12 %, WRN-16-4 (256) -1.1 % per step; beyond, the one kernel was no gain over
      // the three it replaces (LeNet, 500 features: +1.9 %; WRN-28-10, 640: +0.9 %)
      last.head = true;
      N.head_op = (int)N.ops.size() - 1;
    }
    // ... or a global average pool over class maps: pooling, loss and the pooling's backward pass in one kernel
    if (fused_head && last.type == OP_GAP && last.out == N.t_logits && N.tensors[last.out].f32 &&
        N.tensors[last.in].C <= 16) {
      last.head = true;
      N.head_op = (int)N.ops.size() - 1;
    }
    N.off_loss_img = N.alloc((int64_t)N.n * N.B * 4);
  }
  // a batch-norm whose input a convolution of the chain writes can get its column sums from that convolution
  for (size_t i = 0; i < N.ops.size(); ++i) {
    if (N.ops[i].type != OP_BNRELU) continue;
    for (size_t j = 0; j < i; ++j)
      if (N.ops[j].type == OP_CONV && N.ops[j].out == N.ops[i].in && !N.ops[j].branch) N.ops[i].stat_src = (int)j;
  }
  // gradients, transposed weights, scratch
  N.leaf_waves = N.max_bn_c > 0 ? 512 : 0;
  int64_t wpartial = 0, wpartial_main = 0, col_bytes = 0;
  for (Op &op : N.ops) {
    if (op.wseg < 0 && op.type == OP_CONV) {
      err = "internal: weight segment not found";
      return false;
    }
    if (op.stride != 1 && op.stride != 2) {
      err = "internal: stride must be 1 or 2";
      return false;
    }
    N.want_grad(op.out);
    if (op.type == OP_CONV) {
      const int64_t wsize = (int64_t)op.Cout * op.R * op.R * op.Cin;
      if (op.need_dx) {
        N.want_grad(op.in);
        if (!op.head) op.wt_off = N.alloc((int64_t)N.n * wsize * N.esize);  // the head kernel reads the weights as they lie
        // few input channels under a wide window (LeNet's second convolution: 20 channels, 25 taps): as a
        // direct implicit GEMM the pass has 20 output columns on 32-wide fp32 MFMA tiles and a contraction
        // of 1250; as dy x W (500 columns, contraction 50) plus a gather over the window it is a fraction
        if (N.dtype == 0 && op.stride == 1 && op.R > 1 && op.Cin <= 32 && op.R * op.R * op.Cin >= 128 &&
            (int64_t)N.B * op.Ho * op.Wo * op.Cin * op.R * op.R < (1LL << 31)) {
          // the products of one image fit in LDS: one kernel, nothing through memory
          static const bool window_kernel = [] {
            const char *e = getenv("PARLE_DGRAD_WINDOW");
            return !(e && atoi(e) == 0);
          }();
          if (window_kernel && dgrad_window_applicable(N.dtype, N.B, op.Hin, op.Win, op.Cin, op.Cout, op.R, op.stride, op.pad))
            op.win = true;
          else
            col_bytes = std::max(col_bytes, (int64_t)N.n * N.B * op.Ho * op.Wo * op.Cin * op.R * op.R * 4), op.col_off = 0;
        }
      }
      // the complete forward geometry: the split plan depends on which kernel variant will run
      ConvGeom g = conv_fwd_geom(ConvShape{N.B, op.Hin, op.Win, op.Cin, op.Cout, op.R, op.stride, op.pad});
      g.leaf_waves = N.leaf_waves;
      int chunk = 0;
      const int S = wgrad_plan(N.dtype, N.n, g, &chunk);
      // (+ Cout: a kernel that also takes the bias gradient puts it behind the weight gradient, see backward())
      if (S > 1 && (int64_t)N.n * S * (wsize + op.Cout) * 4 > (op.need_dx ? wpartial : wpartial_main))
        (op.need_dx ? wpartial : wpartial_main) = (int64_t)N.n * S * (wsize + op.Cout) * 4;
      if ((int64_t)N.B * op.Hin * op.Win * op.Cin >= (1LL << 31) || (int64_t)g.M * op.Cout >= (1LL << 31) ||
          wsize >= (1LL << 31)) {
        err = "a layer exceeds 2^31 elements per replica";
        return false;
      }
    } else {
      N.want_grad(op.in);
    }
  }
  {
    int with_bias = 0, large = 0;
    for (const Op &op : N.ops)
      if (op.type == OP_CONV && op.bseg >= 0 && op.need_dx)
        ++with_bias, large += (int64_t)N.B * op.Ho * op.Wo * op.Cout >= (1LL << 20) ? 1 : 0;
    N.bias_stream = with_bias >= 2 && 2 * large > with_bias;
    const char *e = getenv("PARLE_BIAS_IN_WGRAD");
    N.bias_in_wgrad = !(e && atoi(e) == 0);
    const char *d = getenv("PARLE_IMAGES_DIRECT");
    int readers = 0, reader = -1;
    for (int oi = 0; oi < (int)N.ops.size(); ++oi)
      if (N.ops[oi].in == N.t_images || (N.ops[oi].type == OP_CONV && N.ops[oi].resid == N.t_images)) ++readers, reader = oi;
    if (!(d && atoi(d) == 0) && readers == 1 && N.ops[reader].type == OP_CONV && N.ops[reader].in == N.t_images &&
        !N.ops[reader].need_dx && !N.ops[reader].branch)
      N.images_reader = reader;
  }
  // two kinds of tables: layers whose rows fill whole 16-byte vectors (tiled, vector kernel) and the rest
  for (int vec = 1; vec >= 0; --vec) {
    bool open = false;
    for (const Op &op : N.ops) {
      if (op.type != OP_CONV || !op.need_dx || op.head || op.win) continue;  // these read the weights as they lie
      if ((int)transpose_vector_ok(N.dtype, op.Cout, op.Cin, N.segs[op.wseg].offset) != vec) continue;
      if (!open || N.transposes.back().count == TransposeTable::kMax) {
        N.transposes.emplace_back();
        N.transposes.back().count = 0;
        N.transposes.back().vec = vec;
        open = true;
      }
      TransposeTable &t = N.transposes.back();
      const int i = t.count++;
      t.cout[i] = op.Cout, t.rs[i] = op.R * op.R, t.cin[i] = op.Cin;
      t.src_off[i] = N.segs[op.wseg].offset, t.dst_off[i] = op.wt_off;
      t.tap_major[i] = op.col_off >= 0;
    }
  }
  for (TransposeTable &t : N.transposes) transpose_table_finish(t);
  N.wpartial_bytes = wpartial > 0 ? wpartial : 256;
  N.off_wpartial = N.alloc(N.wpartial_bytes);
  N.off_wpartial_main = N.alloc(wpartial_main > 0 ? wpartial_main : 256);
  N.wpartial_main_bytes = wpartial_main;
  if (col_bytes > 0) {  // one buffer for all layers that take the two-pass route (they run one after the other)
    const int64_t off = N.alloc(col_bytes);
    for (Op &op : N.ops)
      if (op.col_off == 0) op.col_off = off;
  }
  int maxc = N.max_bn_c;
  for (const Op &op : N.ops)
    if (op.type == OP_CONV && op.bseg >= 0 && op.Cout > maxc) maxc = op.Cout;
  N.off_colpartial = N.alloc((int64_t)N.n * 1024 * 2 * (maxc > 0 ? maxc : 1) * 8);
  N.off_colpartial_side = N.alloc((int64_t)N.n * 1024 * 2 * (maxc > 0 ? maxc : 1) * 8);
  N.off_rowcopy = N.alloc(bf ? N.n_pad * 2 : 256);  // bf16 copy of one parameter row for parle_eval
  return true;
}

struct Run {
  Net *N;
  hipStream_t st;
  int n, B;            // replicas and batch of this launch (eval: 1, count)
  const float *params;  // fp32 rows
  const void *params_t; // rows in the activation dtype (== params in fp32 mode)
  int64_t p_rs;
  char *ws;
  const float *images;
  const long long *step_dev;  // inner-step counter (dropout key); NULL outside training
  float *loss_out = nullptr;  // [n] mean losses of this step, or NULL (training with the fused classifier head)
  bool images_direct = false;  // bf16 network whose first layer reads the fp32 images as they lie
  void *tptr(int t) const {
    const Tensor &T = N->tensors[t];
    return T.external || (images_direct && t == N->t_images) ? (void *)images : (void *)(ws + T.off);
  }
  void *gptr(int t) const { return ws + N->tensors[t].goff; }
  int64_t trs(int t) const { return (int64_t)B * N->tensors[t].H * N->tensors[t].W * N->tensors[t].C; }
  const void *wptr(int seg) const { return (const char *)params_t + N->segs[seg].offset * N->esize; }
  const float *fptr(int seg) const { return params + N->segs[seg].offset; }
};

ConvShape shape_of(const Op &op, int B) { return ConvShape{B, op.Hin, op.Win, op.Cin, op.Cout, op.R, op.stride, op.pad}; }
ConvGeom fwd_geom(const Op &op, int B) { return conv_fwd_geom(shape_of(op, B)); }
ConvGeom bwd_geom(const Op &op, int B) { return conv_bwd_geom(shape_of(op, B)); }

// Whether the layer that reads the images can take them as fp32 (forward, and backward-weight when training), for a
// batch of B images per replica.
bool images_direct_ok(const Net &N, int B, bool train, const void *images) {
  if (N.dtype != 1 || N.images_reader < 0) return false;
  const Op &op = N.ops[N.images_reader];
  const ConvGeom g = fwd_geom(op, B);
  GemmIO io{};
  io.ldc = op.Cout;
  io.in_bytes = (long long)B * op.Hin * op.Win * op.Cin * 4;
  if (N.tensors[op.out].f32 || !conv_smallk_applicable(1, g, io) || !aligned_to(images, 4)) return false;
  return !train || wgrad_smallk_applicable(1, g);
}

#define HIP_TRY(expr)                   \
  do {                                  \
    hipError_t _e = (expr);             \
    if (_e != hipSuccess) return _e;    \
  } while (0)

hipError_t forward(const Run &r, bool train, float *bn_stats, const float *bn_eval_row) {
  Net &N = *r.N;
  const int vw = 16 / N.esize;
  const bool branches = train && N.side != nullptr;  // shortcut convolutions beside the chain
  // a shortcut waits until the chain's next convolution has been enqueued (see the note on order in backward())
  int pending = -1;
  // per convolution: partial rows of column sums its epilogue left for the batch-norm that reads its output
  std::vector<int> stat_S(N.ops.size(), 0);
  std::vector<char> wants_stat(N.ops.size(), 0);
  static const bool epilogue_stats = [] {
    const char *e = getenv("PARLE_EPILOGUE_STATS");
    return !(e && atoi(e) == 0);
  }();
  if (train && epilogue_stats)
    for (const Op &op : N.ops)
      if (op.type == OP_BNRELU && op.stat_src >= 0) wants_stat[op.stat_src] = 1;
  auto conv_io = [&](const Op &op, const ConvGeom &g) {
    GemmIO io{};
    io.in = r.tptr(op.in), io.in_rs = r.trs(op.in);
    io.w = r.wptr(op.wseg), io.w_rs = r.p_rs;
    io.out = r.tptr(op.out), io.out_rs = r.trs(op.out), io.ldc = op.Cout;
    io.bias = op.bseg >= 0 ? r.fptr(op.bseg) : nullptr, io.bias_rs = r.p_rs;
    io.resid = op.resid >= 0 ? r.tptr(op.resid) : nullptr, io.resid_rs = op.resid >= 0 ? r.trs(op.resid) : 0;
    io.relu = op.relu;
    io.vecA = (op.Cin % vw == 0) && aligned_to(io.in, 16);
    // 16-byte loads of weight rows.  Global and buffer loads need 4-byte alignment only, which fp32 rows
    // always have; bf16 rows must start on a 16-byte boundary (two-byte offsets would misalign them).
    io.vecB = (g.K % vw == 0) && (N.dtype == 0 || ((N.segs[op.wseg].offset % vw == 0) && (r.p_rs % vw == 0) &&
                                                   aligned_to(io.w, 16)));
    io.in_bytes = io.in_rs * N.esize;
    if (r.images_direct && op.in == N.t_images) io.in_f32 = 1, io.vecA = 0, io.in_bytes = io.in_rs * 4;
    return io;
  };
  auto launch_pending = [&]() -> hipError_t {
    if (pending < 0) return hipSuccess;
    const int pi = pending;
    pending = -1;
    const Op &op = N.ops[pi];
    const ConvGeom g = fwd_geom(op, r.B);
    HIP_TRY(hipStreamWaitEvent(N.side, N.br_fork[pi], 0));
    HIP_TRY(launch_igemm(N.side, N.dtype, N.tensors[op.out].f32, r.n, g, conv_io(op, g)));
    return hipEventRecord(N.br_out[pi], N.side);
  };
  for (int oi = 0; oi < (int)N.ops.size(); ++oi) {
    const Op &op = N.ops[oi];
    switch (op.type) {
      case OP_CONV: {
        if (train && op.head) break;  // runs with the loss (net_train_step)
        const ConvGeom g = fwd_geom(op, r.B);
        if (branches && op.branch) {
          HIP_TRY(launch_pending());
          HIP_TRY(hipEventRecord(N.br_fork[oi], r.st));
          pending = oi;
          break;
        }
        if (branches && op.join >= 0) {
          HIP_TRY(launch_pending());
          HIP_TRY(hipStreamWaitEvent(r.st, N.br_out[op.join], 0));
        }
        GemmIO io = conv_io(op, g);
        // the sums go where the batch-norm's own reduction would put them (room for 1024 partial rows per replica)
        if (wants_stat[oi]) io.stat = (double *)(r.ws + N.off_colpartial), io.stat_capacity = 1024;
        HIP_TRY(launch_igemm(r.st, N.dtype, N.tensors[op.out].f32, r.n, g, io, &stat_S[oi]));
        HIP_TRY(launch_pending());
        break;
      }
      case OP_POOL: {
        const Tensor &ti = N.tensors[op.in];
        HIP_TRY(launch_maxpool_fwd(r.st, N.dtype, r.n, r.B, ti.H, ti.W, ti.C, r.tptr(op.in), r.trs(op.in),
                                   r.tptr(op.out), r.trs(op.out)));
        break;
      }
      case OP_GAP: {
        if (train && op.head) break;  // runs with the loss (net_train_step)
        const Tensor &ti = N.tensors[op.in];
        HIP_TRY(launch_gap_fwd(r.st, N.dtype, N.tensors[op.out].f32, r.n, r.B, ti.H * ti.W, ti.C, r.tptr(op.in),
                               r.trs(op.in), r.tptr(op.out), r.trs(op.out)));
        break;
      }
      case OP_DROP: {
        const Tensor &ti = N.tensors[op.in];
        const float p = N.cfg.dropout;
        const unsigned thresh = train ? (unsigned)floor((double)p * 16777216.0) : 0u;
        HIP_TRY(launch_dropout(r.st, N.dtype, r.n, (long long)r.B * ti.H * ti.W * ti.C, r.tptr(op.in), r.trs(op.in),
                               r.tptr(op.out), r.trs(op.out), nullptr, 0, (unsigned)N.cfg.dropout_seed, r.step_dev,
                               op.site, thresh, train ? 1.0f / (1.0f - p) : 1.0f));
        break;
      }
      case OP_BNRELU: {
        const Tensor &ti = N.tensors[op.in];
        const int M = r.B * ti.H * ti.W;
        float *saved = (float *)(r.ws + op.saved_off);
        if (train) {
          HIP_TRY(launch_bn_train_fwd(r.st, N.dtype, r.n, M, ti.C, r.tptr(op.in), r.trs(op.in), r.fptr(op.gseg),
                                      r.fptr(op.betaseg), r.p_rs, (double *)(r.ws + N.off_colpartial),
                                      op.stat_src >= 0 ? stat_S[op.stat_src] : 0, saved, bn_stats + op.run_off,
                                      N.bn_floats, r.tptr(op.out), r.trs(op.out)));
        } else {
          HIP_TRY(launch_bn_eval_fwd(r.st, N.dtype, M, ti.C, r.tptr(op.in), r.fptr(op.gseg), r.fptr(op.betaseg),
                                     bn_eval_row + op.run_off, saved, r.tptr(op.out)));
        }
        break;
      }
    }
  }
  return launch_pending();
}

hipError_t backward(const Run &r, float *grad) {
  Net &N = *r.N;
  const int vw = 16 / N.esize;
  if (N.side) {
    HIP_TRY(hipStreamWaitEvent(r.st, N.wt_ready, 0));  // transposed on the second stream beside the forward pass
  } else {
    for (const TransposeTable &t : N.transposes)
      HIP_TRY(launch_weight_transpose_all(r.st, N.dtype, r.n, t, r.params_t, r.p_rs, r.ws));
  }
  bool used_side2 = false;
  // input gradient of a convolution (direct kernels) on stream `s`
  auto launch_dgrad = [&](const Op &op, hipStream_t s) -> hipError_t {
    const void *dy = r.gptr(op.dy);
    const int64_t dy_rs = r.trs(op.dy);
    const int64_t wsize = N.segs[op.wseg].size;
    const ConvGeom gb = bwd_geom(op, r.B);
    GemmIO io{};
    io.in = dy, io.in_rs = dy_rs;
    io.w = r.ws + op.wt_off, io.w_rs = wsize;  // transposed once per step, all layers in one launch
    io.out = r.gptr(op.in), io.out_rs = r.trs(op.in), io.ldc = op.Cin;
    io.mask = op.mask_in ? r.tptr(op.in) : nullptr, io.mask_rs = r.trs(op.in);
    io.accumulate = op.dx_accumulate;
    io.vecA = (op.Cout % vw == 0) && aligned_to(dy, 16);
    io.vecB = (gb.K % vw == 0) && (wsize % vw == 0);
    io.in_bytes = io.in_rs * N.esize;
    return launch_igemm(s, N.dtype, false, r.n, gb, io);
  };
  for (int oi = (int)N.ops.size() - 1; oi >= 0; --oi) {
    const Op &op = N.ops[oi];
    switch (op.type) {
      case OP_CONV: {
        const void *dy = r.gptr(op.dy);
        const int64_t dy_rs = r.trs(op.dy);
        ConvGeom gf = fwd_geom(op, r.B);
        gf.leaf_waves = N.leaf_waves;
        // leaves: on the second stream once this op's output gradient is final.  A layer without input
        // gradient (the first one) leaves the first stream idle: its leaves run there, beside whatever the
        // second stream still has queued.
        hipStream_t lst = r.st;
        int64_t colpartial = N.off_colpartial;
        int64_t wpart = N.off_wpartial, wpart_bytes = N.wpartial_bytes;
        const bool fork = N.side && op.need_dx;
        if (fork) {
          HIP_TRY(hipEventRecord(N.dy_ready[oi], r.st));
          lst = N.side, colpartial = N.off_colpartial_side;
        } else if (!op.need_dx) {
          wpart = N.off_wpartial_main, wpart_bytes = N.wpartial_main_bytes;
        }
        // The input gradient is enqueued before the leaves.  The order matters when the step is recorded into a
        // graph: the runtime keeps the first successor of a node on the node's own queue, and a chain that
        // lands behind a branch of leaves waits for them although nothing ties the two.
        if (op.need_dx && !op.branch && !op.head) {
          if (N.side && op.dx_after >= 0) HIP_TRY(hipStreamWaitEvent(r.st, N.br_dx[op.dx_after], 0));
          void *wt = r.ws + op.wt_off;  // transposed once per step, all layers in one launch
          const int64_t wsize = N.segs[op.wseg].size;
          if (op.win) {
            HIP_TRY(launch_dgrad_window(r.st, r.n, r.B, op.Hin, op.Win, op.Cin, op.Cout, op.R, op.pad, (const float *)dy,
                                        dy_rs, (const float *)r.wptr(op.wseg), r.p_rs,
                                        op.mask_in ? (const float *)r.tptr(op.in) : nullptr, r.trs(op.in),
                                        op.dx_accumulate, (float *)r.gptr(op.in), r.trs(op.in)));
          } else if (op.col_off > 0) {
            // col = dy x W: the transposed weights, here ordered [RS][Cin][Cout], are the [N][K] operand as they lie
            const int RS = op.R * op.R, M = r.B * op.Ho * op.Wo, Ncol = op.Cin * RS;
            const ConvGeom gc = conv_fwd_geom(ConvShape{M, 1, 1, op.Cout, Ncol, 1, 1, 0});
            float *col = (float *)(r.ws + op.col_off);
            GemmIO io{};
            io.in = dy, io.in_rs = dy_rs;
            io.w = wt, io.w_rs = wsize;
            io.out = col, io.out_rs = (int64_t)M * Ncol, io.ldc = Ncol;
            io.vecA = (op.Cout % vw == 0) && aligned_to(dy, 16);
            io.vecB = io.vecA;
            io.in_bytes = io.in_rs * N.esize;
            HIP_TRY(launch_igemm(r.st, N.dtype, true, r.n, gc, io));
            HIP_TRY(launch_col2im(r.st, r.n, r.B, op.Hin, op.Win, op.Cin, op.R, op.pad, col, io.out_rs,
                                  op.mask_in ? (const float *)r.tptr(op.in) : nullptr, r.trs(op.in), op.dx_accumulate,
                                  (float *)r.gptr(op.in), r.trs(op.in)));
          } else {
            HIP_TRY(launch_dgrad(op, r.st));
          }
        }
        if (fork) HIP_TRY(hipStreamWaitEvent(N.side, N.dy_ready[oi], 0));

        // the block's shortcut shares this op's output gradient: its input gradient goes first on the second
        // stream (the block's first convolution waits for it), ahead of the weight gradients
        if (op.join >= 0) {
          HIP_TRY(launch_dgrad(N.ops[op.join], lst));
          if (N.side) HIP_TRY(hipEventRecord(N.br_dx[op.join], N.side));
        }
        // the weight-gradient kernel of this layer takes the bias gradient along where it can (it reads all of dy
        // anyway): the bias segment follows the weight segment in the parameter row
        WgradIO io{};
        io.dy = dy, io.dy_rs = dy_rs;
        io.x = r.tptr(op.in), io.x_rs = r.trs(op.in);
        io.pairA = (op.Cout % 2 == 0) && aligned_to(dy, 4);
        io.pairB = (op.Cin % 2 == 0) && aligned_to(io.x, 4);
        io.x_f32 = r.images_direct && op.in == N.t_images;
        const bool bias_in_wgrad = op.bseg >= 0 && N.bias_in_wgrad && wgrad_takes_bias(N.dtype, gf, io) &&
                                   N.segs[op.bseg].offset == N.segs[op.wseg].offset + N.segs[op.wseg].size;
        if (op.bseg >= 0 && !bias_in_wgrad) {
          hipStream_t bst = lst;
          if (fork && N.side2 && N.bias_stream) {
            HIP_TRY(hipStreamWaitEvent(N.side2, N.dy_ready[oi], 0));
            bst = N.side2, used_side2 = true;
          }
          HIP_TRY(launch_bias_grad(bst, N.dtype, r.n, gf.M, op.Cout, dy, dy_rs, (double *)(r.ws + colpartial),
                                   grad + N.segs[op.bseg].offset, r.p_rs));
        }
        {
          int chunk = 0;
          const int S = wgrad_plan(N.dtype, r.n, gf, &chunk);
          io.splits = S, io.chunk = chunk;
          io.with_bias = bias_in_wgrad;
          const int64_t wsize = N.segs[op.wseg].size + (bias_in_wgrad ? op.Cout : 0);  // values per (replica, split)
          if (S == 1) {
            io.out = grad + N.segs[op.wseg].offset, io.out_rs = r.p_rs, io.split_stride = 0;
            HIP_TRY(launch_wgrad(lst, N.dtype, r.n, gf, io));
          } else {
            // never launch with more partials than the plan reserved room for
            if ((int64_t)r.n * S * wsize * 4 > wpart_bytes) return hipErrorInvalidValue;
            io.out = (float *)(r.ws + wpart), io.out_rs = (int64_t)S * wsize, io.split_stride = wsize;
            HIP_TRY(launch_wgrad(lst, N.dtype, r.n, gf, io));
            HIP_TRY(launch_reduce_partials(lst, r.n, S, wsize, io.out, grad + N.segs[op.wseg].offset, r.p_rs));
          }
        }
        // the mean of the per-image losses is nobody's input: it is taken where the leaves run, after them
        if (op.head && r.loss_out)
          HIP_TRY(launch_loss_mean(lst, r.n, r.B, (const float *)(r.ws + N.off_loss_img), r.loss_out));
        break;
      }
      case OP_POOL: {
        const Tensor &ti = N.tensors[op.in];
        HIP_TRY(launch_maxpool_bwd(r.st, N.dtype, r.n, r.B, ti.H, ti.W, ti.C, r.tptr(op.in), r.trs(op.in),
                                   r.gptr(op.out), r.trs(op.out), r.gptr(op.in), r.trs(op.in), op.pool_relu_mask));
        break;
      }
      case OP_GAP: {
        if (op.head) {
          // the head kernel has written this op's input gradient; the mean of its per-image losses is taken beside
          // the chain
          if (r.loss_out) {
            hipStream_t ls = r.st;
            if (N.side) {
              HIP_TRY(hipEventRecord(N.dy_ready[oi], r.st));
              HIP_TRY(hipStreamWaitEvent(N.side, N.dy_ready[oi], 0));
              ls = N.side;
            }
            HIP_TRY(launch_loss_mean(ls, r.n, r.B, (const float *)(r.ws + N.off_loss_img), r.loss_out));
          }
          break;
        }
        const Tensor &ti = N.tensors[op.in];
        HIP_TRY(launch_gap_bwd(r.st, N.dtype, r.n, r.B, ti.H * ti.W, ti.C, r.gptr(op.out), r.trs(op.out), r.gptr(op.in),
                               r.trs(op.in)));
        break;
      }
      case OP_DROP: {
        const Tensor &ti = N.tensors[op.in];
        const float p = N.cfg.dropout;
        HIP_TRY(launch_dropout(r.st, N.dtype, r.n, (long long)r.B * ti.H * ti.W * ti.C, r.gptr(op.out), r.trs(op.out),
                               r.gptr(op.in), r.trs(op.in), op.drop_relu ? r.tptr(op.in) : nullptr, r.trs(op.in),
                               (unsigned)N.cfg.dropout_seed, r.step_dev, op.site, (unsigned)floor((double)p * 16777216.0),
                               1.0f / (1.0f - p)));
        break;
      }
      case OP_BNRELU: {
        const Tensor &ti = N.tensors[op.in];
        const int M = r.B * ti.H * ti.W;
        HIP_TRY(launch_bn_bwd(r.st, N.dtype, r.n, M, ti.C, r.tptr(op.in), r.trs(op.in), r.gptr(op.out), r.trs(op.out),
                              r.fptr(op.gseg), r.fptr(op.betaseg), r.p_rs, (const float *)(r.ws + op.saved_off),
                              (double *)(r.ws + N.off_colpartial), (float *)(r.ws + op.sums_off),
                              grad + N.segs[op.gseg].offset, grad + N.segs[op.betaseg].offset,
                              op.bn_add >= 0 ? r.gptr(op.bn_add) : nullptr, op.bn_add >= 0 ? r.trs(op.bn_add) : 0,
                              r.gptr(op.in), r.trs(op.in)));
        break;
      }
    }
  }
  if (N.side) {  // join: the update that follows reads every gradient
    HIP_TRY(hipEventRecord(N.side_done, N.side));
    HIP_TRY(hipStreamWaitEvent(r.st, N.side_done, 0));
  }
  if (used_side2) {
    HIP_TRY(hipEventRecord(N.side2_done, N.side2));
    HIP_TRY(hipStreamWaitEvent(r.st, N.side2_done, 0));
  }
  return hipSuccess;
}

// The second stream and its events are made on the first training step outside a stream capture (making
// them is not a stream operation and is not allowed while the calling thread records one).
hipError_t make_side_stream(Net &N, hipStream_t st) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  HIP_TRY(hipStreamIsCapturing(st, &cs));
  if (cs != hipStreamCaptureStatusNone) return hipSuccess;  // this step runs on one stream
  hipStream_t side = nullptr, side2 = nullptr;
  HIP_TRY(hipStreamCreateWithFlags(&side, hipStreamNonBlocking));
  if (hipError_t rc = hipStreamCreateWithFlags(&side2, hipStreamNonBlocking)) {
    (void)hipStreamDestroy(side);
    return rc;
  }
  // per op: output gradient final; per shortcut op three more (see Net); one for the join at the end
  size_t n_branch = 0;
  for (const Op &op : N.ops) n_branch += op.branch ? 1 : 0;
  std::vector<hipEvent_t> ev(N.ops.size() + 3 * n_branch + 4, nullptr);
  for (hipEvent_t &e : ev) {
    if (hipError_t rc = hipEventCreateWithFlags(&e, hipEventDisableTiming)) {
      for (hipEvent_t d : ev)
        if (d) (void)hipEventDestroy(d);
      (void)hipStreamDestroy(side);
      (void)hipStreamDestroy(side2);
      return rc;
    }
  }
  N.side_done = ev.back(), ev.pop_back();
  N.side2_done = ev.back(), ev.pop_back();
  N.step_begin = ev.back(), ev.pop_back();
  N.wt_ready = ev.back(), ev.pop_back();
  N.br_fork.assign(N.ops.size(), nullptr), N.br_out.assign(N.ops.size(), nullptr), N.br_dx.assign(N.ops.size(), nullptr);
  for (size_t oi = 0; oi < N.ops.size(); ++oi) {
    if (!N.ops[oi].branch) continue;
    N.br_fork[oi] = ev.back(), ev.pop_back();
    N.br_out[oi] = ev.back(), ev.pop_back();
    N.br_dx[oi] = ev.back(), ev.pop_back();
  }
  N.dy_ready = ev;
  N.side = side;
  N.side2 = side2;
  return hipSuccess;
}

}  // namespace

Net *net_create(const parle_config &cfg, const Arch &a, const std::vector<Segment> &segs, int64_t n_pad,
                std::string &err) {
  Net *N = new Net();
  N->cfg = cfg, N->arch = a, N->segs = segs, N->n_pad = n_pad;
  N->n = cfg.n_replicas, N->B = cfg.batch, N->dtype = cfg.compute_bf16 ? 1 : 0, N->esize = cfg.compute_bf16 ? 2 : 4;
  if ((int64_t)N->B * a.H * a.W * a.C >= (1LL << 31)) {
    err = "batch * image size exceeds 2^31 elements";
    delete N;
    return nullptr;
  }
  if (!build_plan(*N, err)) {
    delete N;
    return nullptr;
  }
  if (const char *e = getenv("PARLE_OVERLAP_WGRAD")) N->overlap = atoi(e) != 0;
  return N;
}

void net_destroy(Net *net) { delete net; }
int64_t net_workspace_bytes(const Net *net) { return net->ws_bytes; }
int64_t net_bn_floats_per_replica(const Net *net) { return net->bn_floats; }
int64_t net_forward_flops_per_image(const Net *net) {
  int64_t f = 0;
  for (const Op &op : net->ops)
    if (op.type == OP_CONV) f += 2LL * op.Ho * op.Wo * op.Cout * op.R * op.R * op.Cin;
  return f;
}

hipError_t net_train_step(Net *net, hipStream_t st, const float *params, const void *params_bf16, float *grad,
                          float *bn_stats, void *workspace, const float *images, const int32_t *labels,
                          float *loss_dev, const long long *step_dev) {
  Net &N = *net;
  if (N.cfg.dropout > 0.f && !step_dev) return hipErrorInvalidValue;
  if (N.overlap && !N.side) HIP_TRY(make_side_stream(N, st));
  Run r{net, st, N.n, N.B, params, N.dtype ? params_bf16 : (const void *)params, N.n_pad, (char *)workspace, images,
        step_dev};
  r.images_direct = images_direct_ok(N, N.B, true, images);
  if (N.dtype == 1 && !r.images_direct) {
    const Tensor &ti = N.tensors[N.t_images];
    HIP_TRY(launch_convert(st, 1, images, r.ws + ti.off, (long long)N.n * N.B * ti.H * ti.W * ti.C));
  }
  if (N.side) HIP_TRY(hipEventRecord(N.step_begin, st));
  HIP_TRY(forward(r, true, bn_stats, nullptr));
  if (N.side) {
    // the transposed weights are read by the backward pass only: the second stream makes them beside the forward
    // pass (enqueued after it, see the note on order in backward(); they wait for the start of the step only)
    HIP_TRY(hipStreamWaitEvent(N.side, N.step_begin, 0));
    for (const TransposeTable &t : N.transposes)
      HIP_TRY(launch_weight_transpose_all(N.side, N.dtype, r.n, t, r.params_t, r.p_rs, r.ws));
    HIP_TRY(hipEventRecord(N.wt_ready, N.side));
  }
  const Tensor &tl = N.tensors[N.t_logits];
  if (N.head_op >= 0 && N.ops[N.head_op].type == OP_GAP) {
    const Op &op = N.ops[N.head_op];
    const Tensor &ti = N.tensors[op.in];
    HIP_TRY(launch_gap_head(st, N.dtype, N.n, N.B, ti.H * ti.W, ti.C, r.tptr(op.in), r.trs(op.in), labels,
                            (float *)(r.ws + N.off_loss_img), r.gptr(N.t_logits), r.trs(N.t_logits), r.gptr(op.in),
                            r.trs(op.in)));
    r.loss_out = loss_dev;
  } else if (N.head_op >= 0) {
    const Op &op = N.ops[N.head_op];
    float *loss_img = (float *)(r.ws + N.off_loss_img);
    HIP_TRY(launch_fc_head(st, N.dtype, N.n, N.B, op.Cin, op.Cout, r.tptr(op.in), r.trs(op.in), r.wptr(op.wseg), r.p_rs,
                           op.bseg >= 0 ? r.fptr(op.bseg) : nullptr, r.p_rs, labels, loss_img, r.gptr(N.t_logits),
                           r.trs(N.t_logits), r.gptr(op.in), r.trs(op.in), op.mask_in));
    r.loss_out = loss_dev;  // averaged beside the chain, see backward()
  } else {
    HIP_TRY(launch_softmax_xent_train(st, N.dtype, N.n, N.B, tl.C, (const float *)r.tptr(N.t_logits),
                                      r.trs(N.t_logits), labels, loss_dev, r.gptr(N.t_logits), r.trs(N.t_logits)));
  }
  return backward(r, grad);
}

hipError_t net_eval(Net *net, hipStream_t st, const float *param_row, const float *bn_row, void *workspace,
                    const float *images, const int32_t *labels, int count, float *loss_sum_dev, int32_t *n_err_dev) {
  Net &N = *net;
  char *ws = (char *)workspace;
  const void *row_t = param_row;
  if (N.dtype == 1) {
    HIP_TRY(launch_convert(st, 1, param_row, ws + N.off_rowcopy, N.n_pad));
    row_t = ws + N.off_rowcopy;
  }
  Run r{net, st, 1, count, param_row, row_t, N.n_pad, ws, images, nullptr};
  r.images_direct = images_direct_ok(N, count, false, images);
  if (N.dtype == 1 && !r.images_direct) {
    const Tensor &ti = N.tensors[N.t_images];
    HIP_TRY(launch_convert(st, 1, images, ws + ti.off, (long long)count * ti.H * ti.W * ti.C));
  }
  HIP_TRY(forward(r, false, nullptr, bn_row));
  const Tensor &tl = N.tensors[N.t_logits];
  return launch_softmax_xent_eval(st, count, tl.C, (const float *)r.tptr(N.t_logits), labels, loss_sum_dev, n_err_dev);
}

hipError_t net_average_bn(Net *net, hipStream_t st, const float *bn_stats, float *out_row) {
  return launch_row_mean(st, net->n, net->bn_floats, bn_stats, net->bn_floats, out_row);
}

hipError_t net_init_bn(Net *net, hipStream_t st, float *bn_stats) {
  // running mean 0, running variance 1, per replica and layer
  for (int rep = 0; rep < net->n; ++rep) {
    for (const Op &op : net->ops) {
      if (op.type != OP_BNRELU) continue;
      const int C = net->tensors[op.in].C;
      float *row = bn_stats + (int64_t)rep * net->bn_floats + op.run_off;
      HIP_TRY(launch_fill(st, row, C, 0.f));
      HIP_TRY(launch_fill(st, row + C, C, 1.f));
    }
  }
  return hipSuccess;
}
