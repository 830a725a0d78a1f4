// Memory-bound layer kernels of the replica-batched networks (all replicas in one launch).
// dtype: 0 = fp32 activations, 1 = bf16 activations.  Tensors are [replica][rows][C] channels-last;
// `rs` arguments are replica strides in elements.
#pragma once
#include "common.h"

// Softmax cross-entropy.  logits fp32 [n][B][C]; labels [n][B].
// train: loss_out[n] = mean loss (may be NULL), dlogits (activation dtype) = (softmax - onehot)/B.
hipError_t launch_softmax_xent_train(hipStream_t st, int dtype, int n, int B, int C, const float *logits,
                                     long long logits_rs, const int32_t *labels, float *loss_out, void *dlogits,
                                     long long dl_rs);
// eval: one parameter set, `count` samples: loss_sum[0] = sum of losses, n_err[0] = #(argmax != label).
// The classifier's last fully connected layer, the mean cross-entropy and the layer's input gradient in one
// launch (training).  feat [n][B][D], w [n][C][D] (activation dtype), bias [n][C] fp32 or NULL, C <= 16 and (C + 8) * D <= 16384.
// Writes dlogits [n][B][C] = (softmax - onehot)/B and dfeat [n][B][D] = dlogits x W (zero where `mask` and
// feat <= 0) in the activation dtype, and the per-image losses loss_img [n][B]; launch_loss_mean averages them.
bool fc_head_applicable(int classes, int features);
hipError_t launch_fc_head(hipStream_t st, int dtype, int n, int B, int D, int C, const void *feat, long long feat_rs,
                          const void *w, long long w_rs, const float *bias, long long bias_rs, const int32_t *labels,
                          float *loss_img, void *dlogits, long long dl_rs, void *dfeat, long long dfeat_rs, bool mask);
// A network that ends in a global average pool over C <= 16 class maps: pooling, loss and the pooling's backward
// pass in one launch.  feat [n][B][HW][C]; writes dlogits [n][B][C], dfeat [n][B][HW][C] = dlogits / HW, loss_img.
hipError_t launch_gap_head(hipStream_t st, int dtype, int n, int B, int HW, int C, const void *feat, long long feat_rs,
                           const int32_t *labels, float *loss_img, void *dlogits, long long dl_rs, void *dfeat,
                           long long dfeat_rs);
hipError_t launch_loss_mean(hipStream_t st, int n, int B, const float *loss_img, float *loss_out);
hipError_t launch_softmax_xent_eval(hipStream_t st, int count, int C, const float *logits, const int32_t *labels,
                                    float *loss_sum, int32_t *n_err);

// 2x2 max-pool, stride 2, floor.  in [n][B,H,W,C] -> out [n][B,H/2,W/2,C].
hipError_t launch_maxpool_fwd(hipStream_t st, int dtype, int n, int B, int H, int W, int C, const void *in,
                              long long in_rs, void *out, long long out_rs);
// din = dout routed to the first maximum of each window, times (in > 0) when relu_mask.
hipError_t launch_maxpool_bwd(hipStream_t st, int dtype, int n, int B, int H, int W, int C, const void *in,
                              long long in_rs, const void *dout, long long dout_rs, void *din, long long din_rs,
                              int relu_mask);

// Global average pool over HW.  in [n][B,HW,C] -> out [n][B,C] (fp32 when out_f32, else activation dtype).
hipError_t launch_gap_fwd(hipStream_t st, int dtype, bool out_f32, int n, int B, int HW, int C, const void *in,
                          long long in_rs, void *out, long long out_rs);
hipError_t launch_gap_bwd(hipStream_t st, int dtype, int n, int B, int HW, int C, const void *dout, long long dout_rs,
                          void *din, long long din_rs);

// Column sums of dy [n][M][C] (bias gradients): partial [n][S][C] doubles, then grad[rep*grad_rs + c].
hipError_t launch_bias_grad(hipStream_t st, int dtype, int n, int M, int C, const void *dy, long long dy_rs,
                            double *partial, float *grad, long long grad_rs);
int colreduce_splits(int n, int M);
// out[rep*out_rs + i] = sum_s partial[(rep*S + s)*len + i], i < len.
hipError_t launch_reduce_partials(hipStream_t st, int n, int S, long long len, const float *partial, float *out,
                                  long long out_rs);

// Batch normalisation (per replica, per channel, over M rows), fused with the ReLU that follows it.
// saved: [n][2][C] fp32 = mean, 1/sqrt(var + eps).  running: [2][C] per replica (mean, var), stride run_rs.
// pre_splits > 0: `partial` already holds [n][pre_splits][2][C] column sums of x and x*x (left there by the
// convolution that wrote x); the reduction pass over x is then skipped.
hipError_t launch_bn_train_fwd(hipStream_t st, int dtype, int n, int M, int C, const void *x, long long x_rs,
                               const float *gamma, const float *beta, long long p_rs, double *partial, int pre_splits,
                               float *saved, float *running, long long run_rs, void *out, long long out_rs);
hipError_t launch_bn_eval_fwd(hipStream_t st, int dtype, int M, int C, const void *x, const float *gamma,
                              const float *beta, const float *running_row, float *saved, void *out);
// dx = BN-ReLU backward of dout (+ add when not NULL); dgamma, dbeta written to grad (fp32, stride p_rs).
hipError_t launch_bn_bwd(hipStream_t st, int dtype, int n, int M, int C, const void *x, long long x_rs,
                         const void *dout, long long dout_rs, const float *gamma, const float *beta, long long p_rs,
                         const float *saved, double *partial, float *sums, float *dgamma, float *dbeta,
                         const void *add, long long add_rs, void *dx, long long dx_rs);

// wt[ci][(r, s, co)] = w[co][(r, s, ci)] for every replica (operand of the backward-data GEMM).
hipError_t launch_weight_transpose(hipStream_t st, int dtype, int n, int Cout, int RS, int Cin, const void *w,
                                   long long w_rs, void *wt, long long wt_rs);
// dst (activation dtype) = src fp32, `count` elements.
// All layers' weight transposes in one launch.  Entry i: weights [Cout][RS][Cin] at element offset
// src_off of a replica's parameter row -> [Cin][RS][Cout] at byte offset dst_off of `dst_base`, one
// copy per replica (replica stride = the layer's weight count).
struct TransposeTable {
  enum { kMax = 40 };
  int count;
  int cout[kMax], rs[kMax], cin[kMax];
  long long src_off[kMax], dst_off[kMax];
  int tap_major[kMax];  // != 0: rows of the result ordered [RS][Cin] instead of [Cin][RS] (two-pass backward-data)
  // vec != 0: every entry has Cout, Cin and src_off that are multiples of the 16-byte vector width of the
  // dtype, one workgroup per 64 x 64 tile, tiles of entry i are workgroups tile_begin[i] .. tile_begin[i+1]-1
  int vec;
  int tile_begin[kMax + 1];
};
// True when a layer may enter a table with vec != 0.
bool transpose_vector_ok(int dtype, int cout, int cin, long long src_off);
// Fills tile_begin (call once the entries of a vec table are complete).
void transpose_table_finish(TransposeTable &tab);
hipError_t launch_weight_transpose_all(hipStream_t st, int dtype, int n, const TransposeTable &tab, const void *params,
                                       long long p_rs, void *dst_base);
// fp32, stride 1: dx[b, h, w, ci] (+)= sum over the window taps of col[(b, h+pad-r, w+pad-s)][(r*R + s)*Cin + ci],
// zeroed where mask <= 0 (mask like dx, may be NULL).  col: [n][B*P*Q][Cin*R*R], P = H + 2 pad - R + 1.
hipError_t launch_col2im(hipStream_t st, int n, int B, int H, int W, int Cin, int R, int pad, const float *col,
                         long long col_rs, const float *mask, long long mask_rs, int accumulate, float *dx,
                         long long dx_rs);
// Dropout with keep-masks from a counter-based hash (definition in parle.h).  `count` elements per replica;
// step_dev holds the inner-step counter.  out = keep ? in * scale : 0; with relu_src the result is also
// zeroed where relu_src <= 0 (backward through a ReLU that the dropout followed).  thresh = 0 copies.
hipError_t launch_dropout(hipStream_t st, int dtype, int n, long long count, const void *in, long long in_rs, void *out,
                          long long out_rs, const void *relu_src, long long relu_rs, unsigned seed,
                          const long long *step_dev, int site, unsigned thresh, float scale);
hipError_t launch_convert(hipStream_t st, int dtype, const float *src, void *dst, long long count);
hipError_t launch_fill(hipStream_t st, float *dst, long long count, float value);
// out[i] = mean over replicas of in[rep*rs + i].
hipError_t launch_row_mean(hipStream_t st, int n, long long len, const float *in, long long rs, float *out);
