// C ABI of the Parle step: configuration checks, call ordering, scoping rule (9), and the
// sequencing of the kernels.  All arithmetic on tensors happens in the kernels.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <string>

#include "net.h"

struct parle_ctx {
  parle_config cfg;
  parle_buffers buf;
  parle_sizes sizes;
  Arch arch;
  Net *net = nullptr;
  hipStream_t stream = nullptr;
  int64_t k = 0, outer_done = 0, inner_since_outer = 0;
  double g = 0.0, r = 0.0;  // multipliers 1/gamma, 1/rho of rule (9), kept in double on the host
  std::string err;
  // graph replay of an inner block: the library's own stream, the events that tie it to the caller's
  // stream, the instantiated graph and the arguments it was recorded for
  hipStream_t gstream = nullptr;
  hipEvent_t ev_in = nullptr, ev_out = nullptr;
  hipGraphExec_t gexec = nullptr;
  const void *gk_images = nullptr, *gk_labels = nullptr, *gk_loss = nullptr;
  int32_t gk_steps = 0;
};

void parle_internal_set_error(const std::string &msg);

namespace {

constexpr int64_t kRowAlign = 1024;      // elements: every replica row starts 4 KiB aligned
constexpr int64_t kHeaderBytes = 65536;  // front of the workspace: spread partials and result scalars
constexpr int64_t kScalarOff = 32768;
constexpr int64_t kCouplingOff = kScalarOff + 64;  // {g, r} for launches that read them from memory
constexpr int64_t kStepOff = kScalarOff + 128;     // inner-step counter k that the dropout masks are keyed by

thread_local std::string g_init_err;

parle_status fail(parle_ctx *ctx, parle_status s, const std::string &msg) {
  if (ctx)
    ctx->err = msg;
  else
    g_init_err = msg;
  return s;
}

}  // namespace

void parle_internal_set_error(const std::string &msg) { g_init_err = msg; }

namespace {

parle_status check_config(const parle_config *cfg, Arch &arch, std::string &msg) {
  if (!cfg) {
    msg = "null config";
    return PARLE_EINVAL;
  }
  if (cfg->n_replicas < 1 || cfg->n_replicas > 65535) {
    msg = "n_replicas must be in [1, 65535]";
    return PARLE_EINVAL;
  }
  if (cfg->L < 1) {
    msg = "L must be >= 1";
    return PARLE_EINVAL;
  }
  if (cfg->model != PARLE_MODEL_FLAT && (cfg->batch < 1 || cfg->batch > 65536)) {
    msg = "batch must be in [1, 65536]";
    return PARLE_EINVAL;
  }
  if (cfg->model == PARLE_MODEL_FLAT && cfg->n_params < 1) {
    msg = "FLAT model needs n_params >= 1";
    return PARLE_EINVAL;
  }
  const float fl[] = {cfg->eta_inner, cfg->eta_outer, cfg->momentum, cfg->alpha, cfg->weight_decay,
                      cfg->gamma0,    cfg->rho0,      cfg->gamma_max, cfg->rho_max};
  for (float f : fl)
    if (!isfinite(f) || f < 0.f) {
      msg = "step sizes, momentum, alpha, weight decay and couplings must be finite and >= 0";
      return PARLE_EINVAL;
    }
  if (cfg->alpha > 1.f || cfg->momentum >= 1.f) {
    msg = "alpha must be <= 1 and momentum < 1";
    return PARLE_EINVAL;
  }
  if (cfg->scoping_B < 0 || (cfg->xa_mode | 1) != 1 || (cfg->xref_mode | 1) != 1 || (cfg->fuse_outer | 1) != 1 ||
      (cfg->compute_bf16 | 1) != 1 || (cfg->reset_flags & ~3)) {
    msg = "scoping_B, xa_mode, xref_mode, fuse_outer, compute_bf16 or reset_flags out of range";
    return PARLE_EINVAL;
  }
  if ((cfg->algorithm | 1) != 1 || (cfg->graph_block | 1) != 1) {
    msg = "algorithm or graph_block out of range";
    return PARLE_EINVAL;
  }
  if (!(cfg->dropout >= 0.f) || !(cfg->dropout < 1.f) || (cfg->lenet_bn | 1) != 1) {
    msg = "dropout must be in [0, 1), lenet_bn 0 or 1";
    return PARLE_EINVAL;
  }
  if (cfg->graph_block && cfg->model == PARLE_MODEL_FLAT) {
    msg = "graph_block needs a network model";
    return PARLE_EINVAL;
  }
  if (cfg->xref_mode == 1 && cfg->fuse_outer == 0) {
    // the lagged reference needs old and new reference at once: only the fused kernel does that
    msg = "xref_mode = 1 requires fuse_outer = 1";
    return PARLE_EINVAL;
  }
  if (!resolve_arch(*cfg, arch, msg)) return PARLE_EINVAL;
  return PARLE_OK;
}

int64_t bn_average_bytes(const Net *net) {
  return net ? (net_bn_floats_per_replica(net) * (int64_t)sizeof(float) + 255) / 256 * 256 : 0;
}

parle_status compute_sizes(const parle_config *cfg, parle_sizes *out, Arch &arch, std::vector<Segment> &segs,
                           Net **net_out, std::string &msg) {
  if (parle_status s = check_config(cfg, arch, msg)) return s;
  memset(out, 0, sizeof(*out));
  if (cfg->model == PARLE_MODEL_FLAT) {
    out->n_params = cfg->n_params;
  } else {
    segs = build_layout(arch);
    out->n_params = segs.empty() ? 0 : segs.back().offset + segs.back().size;
    out->n_segments = (int32_t)segs.size();
    out->image_elems = arch.H * arch.W * arch.C;
  }
  out->n_pad = (out->n_params + kRowAlign - 1) / kRowAlign * kRowAlign;
  if ((double)out->n_pad * cfg->n_replicas >= 1099511627776.0) {
    msg = "n_replicas * n_pad must stay below 2^40 elements";
    return PARLE_ESIZE;
  }
  out->state_bytes = out->n_pad * cfg->n_replicas * (int64_t)sizeof(float);
  out->shadow_bytes = cfg->compute_bf16 ? out->n_pad * cfg->n_replicas * 2 : 0;
  out->workspace_bytes = kHeaderBytes;
  if (cfg->model != PARLE_MODEL_FLAT) {
    Net *net = net_create(*cfg, arch, segs, out->n_pad, msg);
    if (!net) return PARLE_EINVAL;
    out->workspace_bytes += bn_average_bytes(net) + net_workspace_bytes(net);
    out->bn_bytes = net_bn_floats_per_replica(net) * cfg->n_replicas * (int64_t)sizeof(float);
    out->forward_flops_per_image = net_forward_flops_per_image(net);
    if (net_out)
      *net_out = net;
    else
      net_destroy(net);
  }
  return PARLE_OK;
}

parle_status hip_fail(parle_ctx *ctx, hipError_t e, const char *what) {
  return fail(ctx, PARLE_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

// Workspace: header | replica-averaged BN running statistics (evaluation at the reference) | the network's own
float *bn_average_dev(parle_ctx *ctx) { return (float *)((char *)ctx->buf.workspace + kHeaderBytes); }
void *net_ws(parle_ctx *ctx) { return (char *)ctx->buf.workspace + kHeaderBytes + bn_average_bytes(ctx->net); }

float *coupling_dev(parle_ctx *ctx) {
  return ctx->cfg.graph_block ? (float *)((char *)ctx->buf.workspace + kCouplingOff) : nullptr;
}

// The dropout kernels read k from device memory (a captured launch cannot change its arguments); it is
// advanced by a one-thread kernel after every inner step.
long long *step_dev(parle_ctx *ctx) {
  return ctx->cfg.dropout > 0.f && ctx->cfg.model != PARLE_MODEL_FLAT ? (long long *)((char *)ctx->buf.workspace + kStepOff)
                                                                       : nullptr;
}
parle_status push_step(parle_ctx *ctx) {
  if (!step_dev(ctx)) return PARLE_OK;
  return parle_internal_set_step(ctx->stream, step_dev(ctx), ctx->k);
}

// g, r changed on the host: refresh the copy that captured launches read
parle_status push_coupling(parle_ctx *ctx) {
  if (!ctx->cfg.graph_block) return PARLE_OK;
  return parle_internal_set_coupling(ctx->stream, coupling_dev(ctx), (float)ctx->g, (float)ctx->r);
}

// the replicas that the network is evaluated at and that the spread is measured on
const float *replica_rows(const parle_ctx *ctx) {
  return ctx->cfg.algorithm == PARLE_ALG_ELASTIC ? ctx->buf.y : ctx->buf.x;
}

// One inner step on stream `st`, no bookkeeping: gradient at the replicas, then the fused update.
parle_status enqueue_inner(parle_ctx *ctx, hipStream_t st, const float *images_dev, const int32_t *labels_dev,
                           float *loss_dev) {
  const parle_config &c = ctx->cfg;
  if (c.model != PARLE_MODEL_FLAT) {
    hipError_t e = net_train_step(ctx->net, st, ctx->buf.y, ctx->buf.y_bf16, ctx->buf.grad, (float *)ctx->buf.bn_stats,
                                  net_ws(ctx), images_dev, labels_dev, loss_dev, step_dev(ctx));
    if (e != hipSuccess) return hip_fail(ctx, e, "forward/backward");
    if (step_dev(ctx) && parle_internal_advance_step(st, step_dev(ctx))) return fail(ctx, PARLE_EHIP, "step counter launch failed");
  }
  void *shadow = c.compute_bf16 ? ctx->buf.y_bf16 : nullptr;
  parle_status s;
  if (c.algorithm == PARLE_ALG_ELASTIC)
    s = parle_internal_elastic_step(st, c.n_replicas, ctx->sizes.n_pad, ctx->buf.grad, ctx->buf.y, ctx->buf.vy,
                                    ctx->buf.x_ref, shadow, c.eta_inner, c.eta_outer, c.momentum, c.weight_decay,
                                    (float)ctx->r, coupling_dev(ctx));
  else
    s = parle_internal_inner_update(st, c.n_replicas, ctx->sizes.n_pad, ctx->buf.grad, ctx->buf.x, ctx->buf.y,
                                    ctx->buf.vy, ctx->buf.z, shadow, c.eta_inner, c.momentum, c.alpha, c.weight_decay,
                                    (float)ctx->g, coupling_dev(ctx));
  if (s) return fail(ctx, s, "update launch failed");
  return PARLE_OK;
}

void drop_graph(parle_ctx *ctx) {
  if (ctx->gexec) (void)hipGraphExecDestroy(ctx->gexec);
  ctx->gexec = nullptr;
}

}  // namespace

extern "C" {

parle_status parle_query_sizes(const parle_config *cfg, parle_sizes *out) {
  if (!out) return fail(nullptr, PARLE_EINVAL, "null output");
  Arch arch;
  std::vector<Segment> segs;
  std::string msg;
  parle_status s = compute_sizes(cfg, out, arch, segs, nullptr, msg);
  return s ? fail(nullptr, s, msg) : PARLE_OK;
}

parle_status parle_query_layout(const parle_config *cfg, int32_t index, parle_segment *out) {
  if (!out) return fail(nullptr, PARLE_EINVAL, "null output");
  Arch arch;
  std::string msg;
  if (parle_status s = check_config(cfg, arch, msg)) return fail(nullptr, s, msg);
  std::vector<Segment> segs = build_layout(arch);
  if (index < 0 || index >= (int32_t)segs.size()) return fail(nullptr, PARLE_EINVAL, "segment index out of range");
  const Segment &sg = segs[index];
  memset(out, 0, sizeof(*out));
  snprintf(out->name, sizeof(out->name), "%s", sg.name.c_str());
  out->offset = sg.offset;
  out->size = sg.size;
  out->kind = sg.kind;
  for (int i = 0; i < 4; ++i) out->shape[i] = sg.shape[i];
  out->fan_in = sg.fan_in;
  return PARLE_OK;
}

parle_status parle_init(const parle_config *cfg, const parle_buffers *buf, void *hip_stream, parle_ctx **out) {
  if (!out) return fail(nullptr, PARLE_EINVAL, "null output");
  *out = nullptr;
  if (!buf) return fail(nullptr, PARLE_EINVAL, "null buffers");
  parle_ctx *ctx = new (std::nothrow) parle_ctx();
  if (!ctx) return fail(nullptr, PARLE_ENOMEM, "host allocation failed");
  std::vector<Segment> segs;
  std::string msg;
  if (parle_status s = compute_sizes(cfg, &ctx->sizes, ctx->arch, segs, &ctx->net, msg)) {
    delete ctx;
    return fail(nullptr, s, msg);
  }
  ctx->cfg = *cfg;
  ctx->buf = *buf;
  ctx->stream = (hipStream_t)hip_stream;
  auto bail = [&](parle_status s, const std::string &m) {
    net_destroy(ctx->net);
    delete ctx;
    return fail(nullptr, s, m);
  };
  const void *need[] = {buf->x, buf->y, buf->z, buf->vy, buf->vx, buf->grad, buf->x_ref, buf->workspace};
  for (const void *p : need) {
    if (!p) return bail(PARLE_EINVAL, "a required device buffer is NULL");
    if (!aligned_to(p, 256)) return bail(PARLE_EALIGN, "device buffers must be 256-byte aligned");
  }
  if (cfg->compute_bf16 && (!buf->y_bf16 || !aligned_to(buf->y_bf16, 256)))
    return bail(buf->y_bf16 ? PARLE_EALIGN : PARLE_EINVAL, "compute_bf16 needs a 256-byte aligned y_bf16 buffer");
  if (ctx->sizes.bn_bytes && (!buf->bn_stats || !aligned_to(buf->bn_stats, 256)))
    return bail(buf->bn_stats ? PARLE_EALIGN : PARLE_EINVAL, "this model needs a 256-byte aligned bn_stats buffer");

  ctx->g = cfg->gamma0;
  ctx->r = cfg->rho0;
  const int n = cfg->n_replicas;
  const size_t bytes = (size_t)ctx->sizes.state_bytes;
  hipStream_t st = ctx->stream;
  hipError_t e;
  if ((e = hipMemcpyAsync(buf->y, buf->x, bytes, hipMemcpyDeviceToDevice, st)) != hipSuccess ||
      (e = hipMemcpyAsync(buf->z, buf->x, bytes, hipMemcpyDeviceToDevice, st)) != hipSuccess ||
      (e = hipMemsetAsync(buf->vy, 0, bytes, st)) != hipSuccess ||
      (e = hipMemsetAsync(buf->vx, 0, bytes, st)) != hipSuccess ||
      (e = hipMemsetAsync(buf->grad, 0, bytes, st)) != hipSuccess)
    return bail(PARLE_EHIP, std::string("init copies: ") + hipGetErrorString(e));
  if (parle_status s = parle_k_replica_mean(st, n, ctx->sizes.n_pad, buf->x, buf->x_ref))
    return bail(s, "replica mean launch failed");
  if (cfg->compute_bf16) {
    // y == x and vy == 0, grad == 0: an inner update with step 0 only refreshes the bf16 copy; do it
    // with a dedicated conversion instead so no state tensor is rewritten.
    if (parle_status s = parle_internal_to_bf16(st, buf->y, buf->y_bf16, (int64_t)n * ctx->sizes.n_pad))
      return bail(s, "bf16 conversion launch failed");
  }
  if (ctx->net && ctx->sizes.bn_bytes) {
    if ((e = net_init_bn(ctx->net, st, (float *)buf->bn_stats)) != hipSuccess)
      return bail(PARLE_EHIP, std::string("bn init: ") + hipGetErrorString(e));
  }
  if (push_coupling(ctx)) return bail(PARLE_EHIP, "coupling upload launch failed");
  if (push_step(ctx)) return bail(PARLE_EHIP, "step counter launch failed");
  *out = ctx;
  return PARLE_OK;
}

parle_status parle_inner_step(parle_ctx *ctx, const float *images_dev, const int32_t *labels_dev, float *loss_dev) {
  if (!ctx) return PARLE_EINVAL;
  const parle_config &c = ctx->cfg;
  if (c.model == PARLE_MODEL_FLAT) {
    if (images_dev || labels_dev || loss_dev)
      return fail(ctx, PARLE_EINVAL, "FLAT model takes no images, labels or loss output");
  } else {
    if (!images_dev || !labels_dev) return fail(ctx, PARLE_EINVAL, "images and labels are required");
    if (!aligned_to(images_dev, 16) || !aligned_to(labels_dev, 4) || !aligned_to(loss_dev, 4))
      return fail(ctx, PARLE_EALIGN, "images must be 16-byte aligned, labels and loss 4-byte aligned");
  }
  if (parle_status s = enqueue_inner(ctx, ctx->stream, images_dev, labels_dev, loss_dev)) return s;
  ctx->k += 1;
  ctx->inner_since_outer += 1;
  return PARLE_OK;
}

parle_status parle_inner_block(parle_ctx *ctx, const float *images_dev, const int32_t *labels_dev, int32_t steps,
                               float *loss_dev) {
  if (!ctx) return PARLE_EINVAL;
  const parle_config &c = ctx->cfg;
  if (c.model == PARLE_MODEL_FLAT) return fail(ctx, PARLE_EINVAL, "a block of inner steps needs a network model");
  if (!images_dev || !labels_dev) return fail(ctx, PARLE_EINVAL, "images and labels are required");
  if (steps < 1 || steps > 4096) return fail(ctx, PARLE_EINVAL, "steps must be in [1, 4096]");
  const int64_t img_stride = (int64_t)c.n_replicas * c.batch * ctx->sizes.image_elems;
  const int64_t lab_stride = (int64_t)c.n_replicas * c.batch;
  if (!aligned_to(images_dev, 16) || (img_stride & 3) || !aligned_to(labels_dev, 4) || !aligned_to(loss_dev, 4))
    return fail(ctx, PARLE_EALIGN, "every step's images must be 16-byte aligned, labels and loss 4-byte aligned");
  auto run_steps = [&](hipStream_t st) -> parle_status {
    for (int32_t s = 0; s < steps; ++s)
      if (parle_status rc = enqueue_inner(ctx, st, images_dev + s * img_stride, labels_dev + s * lab_stride,
                                          loss_dev ? loss_dev + (int64_t)s * c.n_replicas : nullptr))
        return rc;
    return PARLE_OK;
  };
  const bool same = ctx->gk_images == images_dev && ctx->gk_labels == labels_dev && ctx->gk_loss == loss_dev &&
                    ctx->gk_steps == steps;
  if (!c.graph_block || !same) {
    // step by step; with graph_block the arguments are remembered and recorded when they come again
    if (parle_status rc = run_steps(ctx->stream)) return rc;
    if (c.graph_block) {
      drop_graph(ctx);
      ctx->gk_images = images_dev, ctx->gk_labels = labels_dev, ctx->gk_loss = loss_dev, ctx->gk_steps = steps;
    }
  } else {
    hipError_t e;
    // each of the three is created once; a call after a failed set-up creates what is still missing
    if ((!ctx->gstream && (e = hipStreamCreateWithFlags(&ctx->gstream, hipStreamNonBlocking)) != hipSuccess) ||
        (!ctx->ev_in && (e = hipEventCreateWithFlags(&ctx->ev_in, hipEventDisableTiming)) != hipSuccess) ||
        (!ctx->ev_out && (e = hipEventCreateWithFlags(&ctx->ev_out, hipEventDisableTiming)) != hipSuccess))
      return hip_fail(ctx, e, "graph stream setup");
    if (!ctx->gexec) {
      if ((e = hipStreamBeginCapture(ctx->gstream, hipStreamCaptureModeThreadLocal)) != hipSuccess)
        return hip_fail(ctx, e, "begin capture");
      const parle_status rc = run_steps(ctx->gstream);
      hipGraph_t graph = nullptr;
      e = hipStreamEndCapture(ctx->gstream, &graph);  // always closes the capture, also after a failed launch
      if (rc || e != hipSuccess) {
        if (graph) (void)hipGraphDestroy(graph);
        return rc ? rc : hip_fail(ctx, e, "end capture");
      }
      e = hipGraphInstantiate(&ctx->gexec, graph, nullptr, nullptr, 0);
      (void)hipGraphDestroy(graph);
      if (e != hipSuccess) {
        ctx->gexec = nullptr;
        return hip_fail(ctx, e, "graph instantiate");
      }
    }
    if ((e = hipEventRecord(ctx->ev_in, ctx->stream)) != hipSuccess ||
        (e = hipStreamWaitEvent(ctx->gstream, ctx->ev_in, 0)) != hipSuccess ||
        (e = hipGraphLaunch(ctx->gexec, ctx->gstream)) != hipSuccess ||
        (e = hipEventRecord(ctx->ev_out, ctx->gstream)) != hipSuccess ||
        (e = hipStreamWaitEvent(ctx->stream, ctx->ev_out, 0)) != hipSuccess)
      return hip_fail(ctx, e, "graph launch");
  }
  ctx->k += steps;
  ctx->inner_since_outer += steps;
  return PARLE_OK;
}

parle_status parle_outer_step(parle_ctx *ctx) {
  if (!ctx) return PARLE_EINVAL;
  if (ctx->inner_since_outer < 1) return fail(ctx, PARLE_ESTATE, "outer step needs an inner step since the last one");
  const parle_config &c = ctx->cfg;
  if (c.algorithm == PARLE_ALG_ELASTIC) {  // Section 2.2 has no outer update: only rho is scoped, by rule (9)
    ctx->outer_done += 1;
    ctx->inner_since_outer = 0;
    if (c.scoping_B > 0) {
      const double q = 1.0 - 1.0 / (2.0 * (double)c.scoping_B);
      ctx->r = fmin(ctx->r / q, (double)c.rho_max);
      if (push_coupling(ctx)) return fail(ctx, PARLE_EHIP, "coupling upload launch failed");
    }
    return PARLE_OK;
  }
  const float cz = c.xa_mode == 0 ? (float)ctx->g : 1.0f;
  parle_status s = PARLE_OK;
  if (!c.fuse_outer) s = parle_k_replica_mean(ctx->stream, c.n_replicas, ctx->sizes.n_pad, ctx->buf.x, ctx->buf.x_ref);
  if (s) return fail(ctx, s, "replica mean launch failed");
  s = parle_k_outer_update(ctx->stream, c.n_replicas, ctx->sizes.n_pad, ctx->buf.x, ctx->buf.z, ctx->buf.vx, ctx->buf.y,
                           ctx->buf.vy, ctx->buf.x_ref, c.compute_bf16 ? ctx->buf.y_bf16 : nullptr, c.eta_outer,
                           c.momentum, cz, (float)ctx->r, c.reset_flags, c.fuse_outer, c.xref_mode);
  if (s) return fail(ctx, s, "outer update launch failed");
  ctx->outer_done += 1;
  ctx->inner_since_outer = 0;
  if (c.scoping_B > 0) {  // rule (9): one factor (1 - 1/(2B)) on gamma, rho per completed outer step
    const double q = 1.0 - 1.0 / (2.0 * (double)c.scoping_B);
    ctx->g = fmin(ctx->g / q, (double)c.gamma_max);
    ctx->r = fmin(ctx->r / q, (double)c.rho_max);
    if (push_coupling(ctx)) return fail(ctx, PARLE_EHIP, "coupling upload launch failed");
  }
  return PARLE_OK;
}

parle_status parle_eval(parle_ctx *ctx, int32_t which, const float *images_dev, const int32_t *labels_dev,
                        int32_t count, float *loss_host, int32_t *n_err_host, float *spread_host) {
  if (!ctx) return PARLE_EINVAL;
  const parle_config &c = ctx->cfg;
  if (which < -1 || which >= c.n_replicas) return fail(ctx, PARLE_EINVAL, "which must be -1 or a replica index");
  char *hdr = (char *)ctx->buf.workspace;
  float *d_spread = (float *)(hdr + kScalarOff);
  float *d_loss = d_spread + 1;
  int32_t *d_nerr = (int32_t *)(d_spread + 2);
  hipError_t e;
  const bool flat = c.model == PARLE_MODEL_FLAT;
  if (flat) {
    if (images_dev || labels_dev || count != 0)
      return fail(ctx, PARLE_EINVAL, "FLAT model evaluates no images (count must be 0)");
  } else {
    if (!images_dev || !labels_dev || !loss_host || !n_err_host)
      return fail(ctx, PARLE_EINVAL, "images, labels and host outputs are required");
    if (count < 1 || (int64_t)count > (int64_t)c.n_replicas * c.batch)
      return fail(ctx, PARLE_EINVAL, "count must be in [1, n_replicas*batch]");
    if (!aligned_to(images_dev, 16)) return fail(ctx, PARLE_EALIGN, "images must be 16-byte aligned");
    const float *row = which < 0 ? ctx->buf.x_ref : replica_rows(ctx) + (int64_t)which * ctx->sizes.n_pad;
    const float *bn_row = nullptr;
    if (ctx->sizes.bn_bytes) {
      const int64_t per = net_bn_floats_per_replica(ctx->net);
      if (which < 0) {
        float *avg = bn_average_dev(ctx);
        if ((e = net_average_bn(ctx->net, ctx->stream, (const float *)ctx->buf.bn_stats, avg)) != hipSuccess)
          return hip_fail(ctx, e, "bn average");
        bn_row = avg;
      } else {
        bn_row = (const float *)ctx->buf.bn_stats + (int64_t)which * per;
      }
    }
    e = net_eval(ctx->net, ctx->stream, row, bn_row, net_ws(ctx), images_dev, labels_dev, count, d_loss, d_nerr);
    if (e != hipSuccess) return hip_fail(ctx, e, "eval forward");
  }
  if (spread_host) {
    parle_status s = parle_k_spread(ctx->stream, c.n_replicas, ctx->sizes.n_pad, replica_rows(ctx), ctx->buf.x_ref,
                                    (double *)hdr, d_spread);
    if (s) return fail(ctx, s, "spread launch failed");
  }
  float h[3] = {0.f, 0.f, 0.f};
  if ((e = hipMemcpyAsync(h, d_spread, sizeof(h), hipMemcpyDeviceToHost, ctx->stream)) != hipSuccess)
    return hip_fail(ctx, e, "result copy");
  if ((e = hipStreamSynchronize(ctx->stream)) != hipSuccess) return hip_fail(ctx, e, "stream synchronize");
  if (spread_host) *spread_host = h[0];
  if (!flat) {
    *loss_host = h[1] / (float)count;
    memcpy(n_err_host, &h[2], sizeof(int32_t));
    if (!isfinite(*loss_host)) return fail(ctx, PARLE_ENONFINITE, "loss is not finite");
  }
  return PARLE_OK;
}

parle_status parle_get_state(const parle_ctx *ctx, int64_t *k, int64_t *outer_done, float *g, float *r) {
  if (!ctx) return PARLE_EINVAL;
  if (k) *k = ctx->k;
  if (outer_done) *outer_done = ctx->outer_done;
  if (g) *g = (float)ctx->g;
  if (r) *r = (float)ctx->r;
  return PARLE_OK;
}

parle_status parle_set_state(parle_ctx *ctx, int64_t k, int64_t outer_done, float g, float r) {
  if (!ctx) return PARLE_EINVAL;
  if (k < 0 || outer_done < 0 || !isfinite(g) || !isfinite(r) || g < 0.f || r < 0.f)
    return fail(ctx, PARLE_EINVAL, "state values must be finite and >= 0");
  if (outer_done > k) return fail(ctx, PARLE_EINVAL, "more outer steps than inner steps");
  ctx->k = k;
  ctx->outer_done = outer_done;
  ctx->g = g;
  ctx->r = r;
  // a resumed run may go straight to an outer step only if the block it interrupts had begun
  // (outer_done <= k, so the quotient test keeps the product inside int64)
  const int64_t L = ctx->cfg.L;
  ctx->inner_since_outer = outer_done <= k / L ? k - outer_done * L : 0;
  if (push_coupling(ctx)) return fail(ctx, PARLE_EHIP, "coupling upload launch failed");
  if (push_step(ctx)) return fail(ctx, PARLE_EHIP, "step counter launch failed");
  return PARLE_OK;
}

const char *parle_last_error(const parle_ctx *ctx) { return ctx ? ctx->err.c_str() : g_init_err.c_str(); }

void parle_destroy(parle_ctx *ctx) {
  if (!ctx) return;
  drop_graph(ctx);
  if (ctx->ev_in) (void)hipEventDestroy(ctx->ev_in);
  if (ctx->ev_out) (void)hipEventDestroy(ctx->ev_out);
  if (ctx->gstream) (void)hipStreamDestroy(ctx->gstream);
  net_destroy(ctx->net);
  delete ctx;
}

}  // extern "C"
