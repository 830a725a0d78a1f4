// Single-kernel C-ABI entry points for the memory-bound layer kernels of the replica-batched networks
// (batch-norm, pooling, dropout, bias gradient, loss), so that each can be checked in isolation on
// caller tensors in both activation formats.
#include <math.h>

#include "nn.h"

namespace {

parle_status check_act(const parle_act_desc *d) {
  if (!d) return PARLE_EINVAL;
  if ((d->dtype | 1) != 1 || d->n < 1 || d->n > 65535 || d->batch < 1 || d->h < 1 || d->w < 1 || d->c < 1)
    return PARLE_EINVAL;
  if ((long long)d->batch * d->h * d->w * d->c >= (1LL << 31)) return PARLE_ESIZE;
  return PARLE_OK;
}

long long rows(const parle_act_desc *d) { return (long long)d->batch * d->h * d->w; }
long long elems(const parle_act_desc *d) { return rows(d) * d->c; }
int64_t reduce_bytes(const parle_act_desc *d) {
  return (int64_t)d->n * colreduce_splits(d->n, (int)rows(d)) * 2 * d->c * (int64_t)sizeof(double);
}
parle_status done(hipError_t e) { return e == hipSuccess ? PARLE_OK : PARLE_EHIP; }

}  // namespace

extern "C" {

int64_t parle_k_layer_scratch_bytes(const parle_act_desc *desc) { return check_act(desc) ? -1 : reduce_bytes(desc); }

parle_status parle_k_bn_forward(void *hip_stream, const parle_act_desc *desc, const void *x, const float *gamma,
                                const float *beta, void *scratch, int64_t scratch_bytes, float *saved, float *running,
                                void *out) {
  if (parle_status s = check_act(desc)) return s;
  if (!x || !gamma || !beta || !scratch || !saved || !out) return PARLE_EINVAL;
  if (!aligned_to(x, 16) || !aligned_to(out, 16) || !aligned_to(scratch, 16)) return PARLE_EALIGN;
  if (scratch_bytes < reduce_bytes(desc)) return PARLE_ESIZE;
  return done(launch_bn_train_fwd((hipStream_t)hip_stream, desc->dtype, desc->n, (int)rows(desc), desc->c, x, elems(desc),
                                  gamma, beta, desc->c, (double *)scratch, 0, saved, running, 2LL * desc->c, out, elems(desc)));
}

parle_status parle_k_bn_backward(void *hip_stream, const parle_act_desc *desc, const void *x, const void *dout,
                                 const float *gamma, const float *beta, const float *saved, const void *add,
                                 void *scratch, int64_t scratch_bytes, float *sums, float *dgamma, float *dbeta, void *dx) {
  if (parle_status s = check_act(desc)) return s;
  if (!x || !dout || !gamma || !beta || !saved || !scratch || !sums || !dgamma || !dbeta || !dx) return PARLE_EINVAL;
  if (!aligned_to(x, 16) || !aligned_to(dout, 16) || !aligned_to(dx, 16) || !aligned_to(add, 16) || !aligned_to(scratch, 16))
    return PARLE_EALIGN;
  if (scratch_bytes < reduce_bytes(desc)) return PARLE_ESIZE;
  return done(launch_bn_bwd((hipStream_t)hip_stream, desc->dtype, desc->n, (int)rows(desc), desc->c, x, elems(desc), dout,
                            elems(desc), gamma, beta, desc->c, saved, (double *)scratch, sums, dgamma, dbeta, add,
                            add ? elems(desc) : 0, dx, elems(desc)));
}

parle_status parle_k_maxpool_forward(void *hip_stream, const parle_act_desc *desc, const void *in, void *out) {
  if (parle_status s = check_act(desc)) return s;
  if (!in || !out || desc->h < 2 || desc->w < 2) return PARLE_EINVAL;
  if (!aligned_to(in, 16) || !aligned_to(out, 16)) return PARLE_EALIGN;
  const long long ors = (long long)desc->batch * (desc->h / 2) * (desc->w / 2) * desc->c;
  return done(launch_maxpool_fwd((hipStream_t)hip_stream, desc->dtype, desc->n, desc->batch, desc->h, desc->w, desc->c, in,
                                 elems(desc), out, ors));
}

parle_status parle_k_maxpool_backward(void *hip_stream, const parle_act_desc *desc, const void *in, const void *dout,
                                      int32_t relu_mask, void *din) {
  if (parle_status s = check_act(desc)) return s;
  if (!in || !dout || !din || desc->h < 2 || desc->w < 2) return PARLE_EINVAL;
  if (!aligned_to(in, 16) || !aligned_to(dout, 16) || !aligned_to(din, 16)) return PARLE_EALIGN;
  const long long ors = (long long)desc->batch * (desc->h / 2) * (desc->w / 2) * desc->c;
  return done(launch_maxpool_bwd((hipStream_t)hip_stream, desc->dtype, desc->n, desc->batch, desc->h, desc->w, desc->c, in,
                                 elems(desc), dout, ors, din, elems(desc), relu_mask != 0));
}

parle_status parle_k_gap_forward(void *hip_stream, const parle_act_desc *desc, int32_t out_f32, const void *in, void *out) {
  if (parle_status s = check_act(desc)) return s;
  if (!in || !out) return PARLE_EINVAL;
  if (!aligned_to(in, 16) || !aligned_to(out, 16)) return PARLE_EALIGN;
  return done(launch_gap_fwd((hipStream_t)hip_stream, desc->dtype, out_f32 != 0, desc->n, desc->batch, desc->h * desc->w,
                             desc->c, in, elems(desc), out, (long long)desc->batch * desc->c));
}

parle_status parle_k_gap_backward(void *hip_stream, const parle_act_desc *desc, const void *dout, void *din) {
  if (parle_status s = check_act(desc)) return s;
  if (!dout || !din) return PARLE_EINVAL;
  if (!aligned_to(dout, 16) || !aligned_to(din, 16)) return PARLE_EALIGN;
  return done(launch_gap_bwd((hipStream_t)hip_stream, desc->dtype, desc->n, desc->batch, desc->h * desc->w, desc->c, dout,
                             (long long)desc->batch * desc->c, din, elems(desc)));
}

parle_status parle_k_dropout(void *hip_stream, const parle_act_desc *desc, const void *in, const void *relu_src,
                             uint32_t seed, const int64_t *step_dev, int32_t site, float p, void *out) {
  if (parle_status s = check_act(desc)) return s;
  if (!in || !out || !step_dev || site < 0 || !(p >= 0.f) || !(p < 1.f)) return PARLE_EINVAL;
  if (!aligned_to(in, 16) || !aligned_to(out, 16) || !aligned_to(relu_src, 16) || !aligned_to(step_dev, 8)) return PARLE_EALIGN;
  return done(launch_dropout((hipStream_t)hip_stream, desc->dtype, desc->n, elems(desc), in, elems(desc), out, elems(desc),
                             relu_src, relu_src ? elems(desc) : 0, seed, (const long long *)step_dev, site,
                             (unsigned)floor((double)p * 16777216.0), 1.0f / (1.0f - p)));
}

parle_status parle_k_bias_grad(void *hip_stream, const parle_act_desc *desc, const void *dy, void *scratch,
                               int64_t scratch_bytes, float *grad) {
  if (parle_status s = check_act(desc)) return s;
  if (!dy || !scratch || !grad) return PARLE_EINVAL;
  if (!aligned_to(dy, 16) || !aligned_to(scratch, 16)) return PARLE_EALIGN;
  if (scratch_bytes < reduce_bytes(desc)) return PARLE_ESIZE;
  return done(launch_bias_grad((hipStream_t)hip_stream, desc->dtype, desc->n, (int)rows(desc), desc->c, dy, elems(desc),
                               (double *)scratch, grad, desc->c));
}

parle_status parle_k_softmax_xent(void *hip_stream, int32_t dtype, int32_t n, int32_t batch, int32_t classes,
                                  const float *logits, const int32_t *labels, float *loss, void *dlogits) {
  if ((dtype | 1) != 1 || n < 1 || n > 65535 || batch < 1 || classes < 1 || !logits || !labels || !dlogits) return PARLE_EINVAL;
  if ((long long)batch * classes >= (1LL << 31)) return PARLE_ESIZE;
  if (!aligned_to(logits, 16) || !aligned_to(dlogits, 16)) return PARLE_EALIGN;
  return done(launch_softmax_xent_train((hipStream_t)hip_stream, dtype, n, batch, classes, logits, (long long)batch * classes,
                                        labels, loss, dlogits, (long long)batch * classes));
}

parle_status parle_k_fc_head(void *hip_stream, int32_t dtype, int32_t n, int32_t batch, int32_t features,
                             int32_t classes, const void *feat, const void *w, const float *bias, const int32_t *labels,
                             int32_t relu_mask, float *loss_img, float *loss, void *dlogits, void *dfeat) {
  if ((dtype | 1) != 1 || n < 1 || n > 65535 || batch < 1 || !fc_head_applicable(classes, features) || !feat || !w ||
      !labels || !loss_img || !dlogits || !dfeat)
    return PARLE_EINVAL;
  if ((long long)batch * features >= (1LL << 31)) return PARLE_ESIZE;
  hipStream_t st = (hipStream_t)hip_stream;
  const hipError_t e = launch_fc_head(st, dtype, n, batch, features, classes, feat, (long long)batch * features, w,
                                      (long long)classes * features, bias, classes, labels, loss_img, dlogits,
                                      (long long)batch * classes, dfeat, (long long)batch * features, relu_mask != 0);
  if (e != hipSuccess) return done(e);
  return loss ? done(launch_loss_mean(st, n, batch, loss_img, loss)) : PARLE_OK;
}

parle_status parle_k_gap_head(void *hip_stream, const parle_act_desc *desc, const void *feat, const int32_t *labels,
                              float *loss_img, float *loss, void *dlogits, void *dfeat) {
  if (parle_status s = check_act(desc)) return s;
  if (!feat || !labels || !loss_img || !dlogits || !dfeat || desc->c > 16) return PARLE_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const hipError_t e = launch_gap_head(st, desc->dtype, desc->n, desc->batch, desc->h * desc->w, desc->c, feat, elems(desc),
                                       labels, loss_img, dlogits, (long long)desc->batch * desc->c, dfeat, elems(desc));
  if (e != hipSuccess) return done(e);
  return loss ? done(launch_loss_mean(st, desc->n, desc->batch, loss_img, loss)) : PARLE_OK;
}

}  // extern "C"
