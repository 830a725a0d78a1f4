// Single-kernel C-ABI entry points for the replica-grouped convolution kernels (forward,
// backward-data, backward-weight), so that each can be checked in isolation on caller tensors.
#include "igemm.h"
#include "nn.h"

namespace {

parle_status check_desc(const parle_conv_desc *d, ConvShape &c) {
  if (!d) return PARLE_EINVAL;
  if ((d->dtype | 1) != 1 || d->n < 1 || d->n > 65535 || d->batch < 1 || d->h < 1 || d->w < 1 || d->cin < 1 ||
      d->cout < 1 || d->k < 1 || (d->stride != 1 && d->stride != 2) || d->pad < 0 || d->pad >= d->k)
    return PARLE_EINVAL;
  if (d->h + 2 * d->pad < d->k || d->w + 2 * d->pad < d->k) return PARLE_EINVAL;
  c = ConvShape{d->batch, d->h, d->w, d->cin, d->cout, d->k, d->stride, d->pad};
  const long long lim = 1LL << 31;
  if ((long long)c.B * c.H * c.W * c.Cin >= lim || (long long)c.B * c.Ho() * c.Wo() * c.Cout >= lim ||
      (long long)c.Cout * c.R * c.R * c.Cin >= lim)
    return PARLE_ESIZE;
  return PARLE_OK;
}

}  // namespace

extern "C" {

parle_status parle_k_conv_forward(void *hip_stream, const parle_conv_desc *desc, const void *x, const void *w,
                                  const float *bias, const void *resid, int32_t relu, void *y) {
  ConvShape c;
  if (parle_status s = check_desc(desc, c)) return s;
  if (!x || !w || !y) return PARLE_EINVAL;
  if (!aligned_to(x, 16) || !aligned_to(w, 16) || !aligned_to(y, 16) || !aligned_to(bias, 4) || !aligned_to(resid, 16))
    return PARLE_EALIGN;
  const int es = desc->dtype ? 2 : 4, vw = 16 / es;
  const ConvGeom g = conv_fwd_geom(c);
  GemmIO io{};
  io.in = x, io.in_rs = (long long)c.B * c.H * c.W * c.Cin;
  io.w = w, io.w_rs = (long long)g.N * g.K;
  io.out = y, io.out_rs = (long long)g.M * g.N, io.ldc = g.N;
  io.bias = bias, io.bias_rs = g.N;
  io.resid = resid, io.resid_rs = io.out_rs;
  io.relu = relu;
  io.vecA = (c.Cin % vw == 0) && (io.in_rs % vw == 0);
  io.vecB = (g.K % vw == 0);
  io.in_bytes = io.in_rs * es;
  return launch_igemm((hipStream_t)hip_stream, desc->dtype, false, desc->n, g, io) == hipSuccess ? PARLE_OK : PARLE_EHIP;
}

parle_status parle_k_conv_forward_colsums(void *hip_stream, const parle_conv_desc *desc, const void *x, const void *w,
                                          const void *resid, void *y, double *partial, int32_t capacity,
                                          int32_t *splits_host) {
  ConvShape c;
  if (parle_status s = check_desc(desc, c)) return s;
  if (!x || !w || !y || !partial || !splits_host || capacity < 1) return PARLE_EINVAL;
  if (!aligned_to(x, 16) || !aligned_to(w, 16) || !aligned_to(y, 16) || !aligned_to(resid, 16) || !aligned_to(partial, 8))
    return PARLE_EALIGN;
  const int es = desc->dtype ? 2 : 4, vw = 16 / es;
  const ConvGeom g = conv_fwd_geom(c);
  GemmIO io{};
  io.in = x, io.in_rs = (long long)c.B * c.H * c.W * c.Cin;
  io.w = w, io.w_rs = (long long)g.N * g.K;
  io.out = y, io.out_rs = (long long)g.M * g.N, io.ldc = g.N;
  io.resid = resid, io.resid_rs = io.out_rs;
  io.vecA = (c.Cin % vw == 0) && (io.in_rs % vw == 0);
  io.vecB = (g.K % vw == 0);
  io.in_bytes = io.in_rs * es;
  io.stat = partial, io.stat_capacity = capacity;
  int S = 0;
  if (launch_igemm((hipStream_t)hip_stream, desc->dtype, false, desc->n, g, io, &S) != hipSuccess) return PARLE_EHIP;
  *splits_host = S;
  return PARLE_OK;
}

parle_status parle_k_conv_backward_data(void *hip_stream, const parle_conv_desc *desc, const void *dy, const void *w,
                                        const void *relu_mask, int32_t accumulate, void *wt_scratch, void *dx) {
  ConvShape c;
  if (parle_status s = check_desc(desc, c)) return s;
  if (!dy || !w || !wt_scratch || !dx) return PARLE_EINVAL;
  if (!aligned_to(dy, 16) || !aligned_to(w, 16) || !aligned_to(dx, 16) || !aligned_to(wt_scratch, 16) ||
      !aligned_to(relu_mask, 16))
    return PARLE_EALIGN;
  const int es = desc->dtype ? 2 : 4, vw = 16 / es;
  hipStream_t st = (hipStream_t)hip_stream;
  const long long wsize = (long long)c.Cout * c.R * c.R * c.Cin;
  if (dgrad_window_applicable(desc->dtype, c.B, c.H, c.W, c.Cin, c.Cout, c.R, c.stride, c.pad)) {
    // the path the network executor takes for such a layer: per-tap products in LDS, weights as they lie
    const long long x_rs = (long long)c.B * c.H * c.W * c.Cin;
    return launch_dgrad_window(st, desc->n, c.B, c.H, c.W, c.Cin, c.Cout, c.R, c.pad, (const float *)dy,
                               (long long)c.B * c.Ho() * c.Wo() * c.Cout, (const float *)w, wsize,
                               (const float *)relu_mask, x_rs, accumulate, (float *)dx, x_rs) == hipSuccess
               ? PARLE_OK
               : PARLE_EHIP;
  }
  if (launch_weight_transpose(st, desc->dtype, desc->n, c.Cout, c.R * c.R, c.Cin, w, wsize, wt_scratch, wsize) !=
      hipSuccess)
    return PARLE_EHIP;
  const ConvGeom g = conv_bwd_geom(c);
  GemmIO io{};
  io.in = dy, io.in_rs = (long long)c.B * c.Ho() * c.Wo() * c.Cout;
  io.w = wt_scratch, io.w_rs = wsize;
  io.out = dx, io.out_rs = (long long)g.M * g.N, io.ldc = g.N;
  io.mask = relu_mask, io.mask_rs = io.out_rs;
  io.accumulate = accumulate;
  io.vecA = (c.Cout % vw == 0) && (io.in_rs % vw == 0);
  io.vecB = (g.K % vw == 0) && (wsize % vw == 0);
  io.in_bytes = io.in_rs * es;
  return launch_igemm(st, desc->dtype, false, desc->n, g, io) == hipSuccess ? PARLE_OK : PARLE_EHIP;
}

}  // extern "C"

namespace {
// dw [n][wsize (+ cout)]: with `took_bias_host` given, the bias gradient follows the weight gradient of each replica
// where the kernel that runs this layer takes it along
parle_status backward_weight(void *hip_stream, const parle_conv_desc *desc, const void *dy, const void *x, float *scratch,
                             int64_t scratch_bytes, float *dw, int32_t *took_bias_host) {
  ConvShape c;
  if (parle_status s = check_desc(desc, c)) return s;
  if (!dy || !x || !dw) return PARLE_EINVAL;
  if (!aligned_to(dy, 16) || !aligned_to(x, 16) || !aligned_to(dw, 16) || !aligned_to(scratch, 16)) return PARLE_EALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  const ConvGeom g = conv_fwd_geom(c);
  WgradIO io{};
  io.dy = dy, io.dy_rs = (long long)g.M * g.N;
  io.x = x, io.x_rs = (long long)c.B * c.H * c.W * c.Cin;
  int chunk = 0;
  const int S = wgrad_plan(desc->dtype, desc->n, g, &chunk);
  io.splits = S, io.chunk = chunk;
  io.pairA = (c.Cout % 2 == 0);
  io.pairB = (c.Cin % 2 == 0);
  io.with_bias = took_bias_host && wgrad_takes_bias(desc->dtype, g, io);
  if (took_bias_host) *took_bias_host = io.with_bias;
  // values a kernel writes per (replica, split), and the caller's row: the bias slots exist in dw whenever the caller
  // asked for this form, and are written only by a kernel that takes the bias along
  const long long wsize = (long long)g.N * g.K + (io.with_bias ? g.N : 0);
  const long long row = (long long)g.N * g.K + (took_bias_host ? g.N : 0);
  if (S == 1) {
    io.out = dw, io.out_rs = row, io.split_stride = 0;
    return launch_wgrad(st, desc->dtype, desc->n, g, io) == hipSuccess ? PARLE_OK : PARLE_EHIP;
  }
  if (!scratch || scratch_bytes < (int64_t)desc->n * S * wsize * 4) return PARLE_ESIZE;
  io.out = scratch, io.out_rs = (long long)S * wsize, io.split_stride = wsize;
  if (launch_wgrad(st, desc->dtype, desc->n, g, io) != hipSuccess) return PARLE_EHIP;
  return launch_reduce_partials(st, desc->n, S, wsize, scratch, dw, row) == hipSuccess ? PARLE_OK : PARLE_EHIP;
}
}  // namespace

extern "C" {

parle_status parle_k_conv_backward_weight(void *hip_stream, const parle_conv_desc *desc, const void *dy, const void *x,
                                          float *scratch, int64_t scratch_bytes, float *dw) {
  return backward_weight(hip_stream, desc, dy, x, scratch, scratch_bytes, dw, nullptr);
}

parle_status parle_k_conv_backward_weight_bias(void *hip_stream, const parle_conv_desc *desc, const void *dy,
                                               const void *x, float *scratch, int64_t scratch_bytes, float *dwb,
                                               int32_t *took_bias_host) {
  if (!took_bias_host) return PARLE_EINVAL;
  return backward_weight(hip_stream, desc, dy, x, scratch, scratch_bytes, dwb, took_bias_host);
}

int64_t parle_k_conv_scratch_bytes(const parle_conv_desc *desc) {
  ConvShape c;
  if (check_desc(desc, c)) return -1;
  const ConvGeom g = conv_fwd_geom(c);
  int chunk = 0;
  const int S = wgrad_plan(desc->dtype, desc->n, g, &chunk);
  return S == 1 ? 0 : (int64_t)desc->n * S * ((int64_t)g.N * g.K + g.N) * 4;
}

}  // extern "C"
