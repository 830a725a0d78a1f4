// Replica-batched network executor: forward, loss, backward for all replicas in grouped launches.
#pragma once
#include <string>
#include <vector>

#include "arch.h"

struct Net;  // host-side plan: tensors, ops, workspace offsets

// Builds the plan on the host (no GPU call).  Returns nullptr and sets err on failure.
Net *net_create(const parle_config &cfg, const Arch &a, const std::vector<Segment> &segs, int64_t n_pad, std::string &err);
void net_destroy(Net *net);
int64_t net_workspace_bytes(const Net *net);
int64_t net_bn_floats_per_replica(const Net *net);
// 2*M*N*K over the contractions of one forward pass, per image
int64_t net_forward_flops_per_image(const Net *net);

// Enqueues forward + loss + backward for all n replicas.  Parameters are read from `params`
// ([n, n_pad] fp32) and, in bf16 mode, from `params_bf16`; gradients go to `grad` ([n, n_pad] fp32,
// every parameter element is overwritten, padding untouched).  `loss_dev` ([n]) may be NULL.
// `step_dev`: the inner-step counter in device memory, read by the dropout masks (NULL without dropout).
hipError_t net_train_step(Net *net, hipStream_t st, const float *params, const void *params_bf16, float *grad,
                          float *bn_stats, void *workspace, const float *images, const int32_t *labels,
                          float *loss_dev, const long long *step_dev);

// Enqueues a forward pass of ONE parameter row over `count` images in evaluation mode (BN uses
// `bn_row`, the statistics of one replica or their average).  Results: loss_sum_dev[0] = sum of
// the per-sample losses, n_err_dev[0] = misclassified count.
hipError_t net_eval(Net *net, hipStream_t st, const float *param_row, const float *bn_row, void *workspace,
                    const float *images, const int32_t *labels, int count, float *loss_sum_dev, int32_t *n_err_dev);

// Averages the per-replica BN running statistics into out_row (device, bn floats per replica).
hipError_t net_average_bn(Net *net, hipStream_t st, const float *bn_stats, float *out_row);
hipError_t net_init_bn(Net *net, hipStream_t st, float *bn_stats);
