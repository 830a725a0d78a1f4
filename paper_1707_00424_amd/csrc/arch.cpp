// Network sizes and parameter packing (host only).  The families are the ones Section 4 of the
// paper trains; the layer lists are stated in parle.h.
#include "arch.h"

namespace {

void add_seg(std::vector<Segment> &v, int64_t &off, const std::string &name, int kind, int s0, int s1, int s2, int s3,
             int fan_in) {
  Segment s;
  s.name = name;
  s.kind = kind;
  s.shape[0] = s0;
  s.shape[1] = s1;
  s.shape[2] = s2;
  s.shape[3] = s3;
  s.size = (int64_t)s0 * (s1 ? s1 : 1) * (s2 ? s2 : 1) * (s3 ? s3 : 1);
  s.offset = off;
  s.fan_in = fan_in;
  off += s.size;
  v.push_back(s);
}

void add_conv(std::vector<Segment> &v, int64_t &off, const std::string &name, int cout, int k, int cin, bool bias) {
  add_seg(v, off, name + ".w", PARLE_SEG_WEIGHT, cout, k, k, cin, k * k * cin);
  if (bias) add_seg(v, off, name + ".b", PARLE_SEG_BIAS, cout, 0, 0, 0, k * k * cin);
}

void add_fc(std::vector<Segment> &v, int64_t &off, const std::string &name, int out, int in) {
  add_seg(v, off, name + ".w", PARLE_SEG_WEIGHT, out, in, 0, 0, in);
  add_seg(v, off, name + ".b", PARLE_SEG_BIAS, out, 0, 0, 0, in);
}

void add_bn(std::vector<Segment> &v, int64_t &off, const std::string &name, int c) {
  add_seg(v, off, name + ".g", PARLE_SEG_BN_GAMMA, c, 0, 0, 0, c);
  add_seg(v, off, name + ".b", PARLE_SEG_BN_BETA, c, 0, 0, 0, c);
}

int pick(int v, int dflt) { return v > 0 ? v : dflt; }

}  // namespace

bool resolve_arch(const parle_config &cfg, Arch &a, std::string &msg) {
  a = Arch();
  a.model = cfg.model;
  if (cfg.in_h < 0 || cfg.in_w < 0 || cfg.in_c < 0 || cfg.n_classes < 0) {
    msg = "negative input size";
    return false;
  }
  for (int i = 0; i < 4; ++i)
    if (cfg.arch[i] < 0) {
      msg = "negative arch[] entry";
      return false;
    }
  switch (cfg.model) {
    case PARLE_MODEL_FLAT:
      return true;
    case PARLE_MODEL_MLP:
      a.H = pick(cfg.in_h, 28), a.W = pick(cfg.in_w, 28), a.C = pick(cfg.in_c, 1), a.classes = pick(cfg.n_classes, 10);
      a.a0 = pick(cfg.arch[0], 128);
      return true;
    case PARLE_MODEL_LENET: {
      a.H = pick(cfg.in_h, 28), a.W = pick(cfg.in_w, 28), a.C = pick(cfg.in_c, 1), a.classes = pick(cfg.n_classes, 10);
      a.a0 = pick(cfg.arch[0], 20), a.a1 = pick(cfg.arch[1], 50), a.a2 = pick(cfg.arch[2], 5), a.a3 = pick(cfg.arch[3], 500);
      a.bn = cfg.lenet_bn;
      const int k = a.a2;
      const int h1 = (a.H - k + 1) / 2, w1 = (a.W - k + 1) / 2;
      const int h2 = (h1 - k + 1) / 2, w2 = (w1 - k + 1) / 2;
      if (a.H < k || a.W < k || h1 < k || w1 < k || h2 < 1 || w2 < 1) {
        msg = "LeNet: input too small for two k x k convolutions with 2x2 pooling";
        return false;
      }
      return true;
    }
    case PARLE_MODEL_ALLCNN_C:
      a.H = pick(cfg.in_h, 32), a.W = pick(cfg.in_w, 32), a.C = pick(cfg.in_c, 3), a.classes = pick(cfg.n_classes, 10);
      a.a0 = pick(cfg.arch[0], 96), a.a1 = pick(cfg.arch[1], 192);
      return true;
    case PARLE_MODEL_WRN:
      a.H = pick(cfg.in_h, 32), a.W = pick(cfg.in_w, 32), a.C = pick(cfg.in_c, 3), a.classes = pick(cfg.n_classes, 10);
      a.a0 = pick(cfg.arch[0], 16), a.a1 = pick(cfg.arch[1], 4), a.a2 = pick(cfg.arch[2], 2);
      return true;
    default:
      msg = "unknown model";
      return false;
  }
}

std::vector<WrnBlock> wrn_block_list(const Arch &a) {
  std::vector<WrnBlock> out;
  int cin = a.a0;
  for (int gi = 0; gi < 3; ++gi) {
    const int width = a.a0 * a.a1 * (1 << gi);
    for (int bi = 0; bi < a.a2; ++bi) {
      WrnBlock b;
      b.name = "g" + std::to_string(gi + 1) + "b" + std::to_string(bi + 1);
      b.cin = cin;
      b.cout = width;
      b.stride = (bi == 0 && gi > 0) ? 2 : 1;
      b.has_sc = (b.cin != b.cout) || b.stride != 1;
      out.push_back(b);
      cin = width;
    }
  }
  return out;
}

std::vector<Segment> build_layout(const Arch &a) {
  std::vector<Segment> v;
  int64_t off = 0;
  switch (a.model) {
    case PARLE_MODEL_MLP:
      add_fc(v, off, "fc1", a.a0, a.H * a.W * a.C);
      add_fc(v, off, "fc2", a.classes, a.a0);
      break;
    case PARLE_MODEL_LENET: {
      const int k = a.a2;
      const int h1 = (a.H - k + 1) / 2, w1 = (a.W - k + 1) / 2;
      const int h2 = (h1 - k + 1) / 2, w2 = (w1 - k + 1) / 2;
      add_conv(v, off, "conv1", a.a0, k, a.C, true);
      if (a.bn) add_bn(v, off, "bn1", a.a0);
      add_conv(v, off, "conv2", a.a1, k, a.a0, true);
      if (a.bn) add_bn(v, off, "bn2", a.a1);
      add_fc(v, off, "fc1", a.a3, h2 * w2 * a.a1);
      if (a.bn) add_bn(v, off, "bn3", a.a3);
      add_fc(v, off, "fc2", a.classes, a.a3);
      break;
    }
    case PARLE_MODEL_ALLCNN_C: {
      const int ca = a.a0, cb = a.a1;
      const int cin[9] = {a.C, ca, ca, ca, cb, cb, cb, cb, cb};
      const int cout[9] = {ca, ca, ca, cb, cb, cb, cb, cb, a.classes};
      const int ks[9] = {3, 3, 3, 3, 3, 3, 3, 1, 1};
      for (int i = 0; i < 9; ++i) add_conv(v, off, "conv" + std::to_string(i + 1), cout[i], ks[i], cin[i], true);
      break;
    }
    case PARLE_MODEL_WRN: {
      add_conv(v, off, "conv1", a.a0, 3, a.C, false);
      for (const WrnBlock &b : wrn_block_list(a)) {
        add_bn(v, off, b.name + ".bn1", b.cin);
        add_conv(v, off, b.name + ".conv1", b.cout, 3, b.cin, false);
        add_bn(v, off, b.name + ".bn2", b.cout);
        add_conv(v, off, b.name + ".conv2", b.cout, 3, b.cout, false);
        if (b.has_sc) add_conv(v, off, b.name + ".sc", b.cout, 1, b.cin, false);
      }
      const int cl = a.a0 * a.a1 * 4;
      add_bn(v, off, "bn_out", cl);
      add_fc(v, off, "fc", a.classes, cl);
      break;
    }
    default:
      break;
  }
  return v;
}

int find_segment(const std::vector<Segment> &segs, const std::string &name) {
  for (size_t i = 0; i < segs.size(); ++i)
    if (segs[i].name == name) return (int)i;
  return -1;
}
