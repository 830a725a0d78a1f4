/*
 * parle.h -- C ABI of the Parle replica-coupled training step on one MI355X (gfx950).
 *
 * All n replicas of a network live on one GPU as rows of stacked [n, n_pad] fp32 tensors.
 * The library runs, with hand-written HIP kernels only:
 *   - the replica-batched forward / loss / backward that yields grad f(y^a) of update (8a),
 *   - the fused inner update: (8a) with Nesterov momentum and the running average (8b),
 *   - the replica mean: (8d) with eta'' = rho/n (Section 3.1),
 *   - the fused outer update: (8c) with Nesterov momentum and the reset y^a <- x^a,
 *   - the scoping rule (9) on the host,
 *   - as a variant, Elastic-SGD (Section 2.2) with scoping on rho (algorithm = 1).
 * Equation, section and remark numbers refer to "Parle: parallelizing stochastic gradient
 * descent" (arXiv 1707.00424).
 *
 * COUPLING CONVENTION.  The paper writes the couplings as 1/gamma and 1/rho and decays gamma, rho.
 * This ABI uses the multipliers g = 1/gamma, r = 1/rho: the proximal force of (8a) is
 * g * (y - x^a), the elastic force of (8c) is r * (x^a - x_ref); scoping makes g and r grow
 * up to gamma_max, rho_max.
 *
 * GENERAL RULES.  Plain C types only.  Every function returns a parle_status and never throws.
 * Pointers named "dev" are DEVICE pointers owned by the caller (any allocator; PyTorch tensors in
 * the bundled binding); pointers named "host" are host pointers.  The library allocates no
 * device memory and frees none.  All device work is ordered on the HIP stream given at init and is
 * asynchronous unless stated: a context of a network model owns up to three more streams of default priority
 * (weight-gradient, bias-gradient and shortcut kernels run beside the chain of the forward and backward pass;
 * blocks of inner steps are replayed from a graph), tied to the init stream by events on both sides, so the caller sees the usual
 * stream order and needs no synchronisation of its own.  Buffers must not alias.  Calls on one context must
 * not overlap in time.  Non-finite values are not trapped by the step calls (parle_eval reports them).
 * Arguments are checked before anything is enqueued: EINVAL, EALIGN, ESIZE and ESTATE leave the
 * context and the device state as they were.  After EHIP from a step call part of the step may have
 * been enqueued: the state tensors are then to be restored from the caller's last copy.
 */
#ifndef PARLE_H
#define PARLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct parle_ctx parle_ctx; /* opaque, host memory, owned by the library */

typedef enum {
  PARLE_ALG_PARLE = 0,   /* updates (8a)-(8d): proximal inner loop, elastic outer step every L steps.
                            n = 1 with rho0 = 0 is Entropy-SGD (Section 2.1, updates (6a)-(6c)). */
  PARLE_ALG_ELASTIC = 1  /* Elastic-SGD, Section 2.2: every step moves all replicas with the elastic
                            force r*(x^a - x) and the reference towards the replica mean.  State: the
                            replicas x^a live in buffers.y (and its bf16 copy), their momentum in
                            buffers.vy, the reference in buffers.x_ref; x is only read by parle_init,
                            z and vx are not touched.  parle_outer_step applies rule (9) to r alone. */
} parle_algorithm;

typedef enum {
  PARLE_OK = 0,
  PARLE_EINVAL = -1,     /* bad argument or configuration field */
  PARLE_ENOMEM = -2,     /* host allocation failed */
  PARLE_EALIGN = -3,     /* a device pointer is not 256-byte aligned */
  PARLE_ESIZE = -4,      /* a size exceeds what the kernels index (see parle_query_sizes) */
  PARLE_EHIP = -5,       /* a HIP call failed; parle_last_error has the text */
  PARLE_ESTATE = -6,     /* call order violated (outer step without an inner step since the last) */
  PARLE_ENONFINITE = -7  /* parle_eval found a NaN/Inf loss */
} parle_status;

typedef enum {
  PARLE_MODEL_FLAT = 0,     /* no network: the caller writes buffers.grad before each inner step */
  PARLE_MODEL_MLP = 1,      /* in - hidden - classes, ReLU;                    arch = {hidden} */
  PARLE_MODEL_LENET = 2,    /* conv-pool-conv-pool-fc-fc;                      arch = {c1, c2, k, fc} */
  PARLE_MODEL_ALLCNN_C = 3, /* All-CNN-C, nine convs + global average pool;    arch = {ca, cb} */
  PARLE_MODEL_WRN = 4       /* pre-activation wide ResNet, depth 6*nb+4;       arch = {base, widen, nb} */
} parle_model;

/*
 * Network definitions (Section 4 names the families; sizes default to the paper's workloads).
 * Activations are channels-last [B, H, W, C].  A conv weight is [Cout, kh, kw, Cin] row-major,
 * an fc weight is [out, in] with the input flattened in (h, w, c) order.  One replica's row of
 * every state tensor packs the segments in execution order, weight before bias, then zero
 * padding up to n_pad; parle_query_layout enumerates the segments.
 *   MLP      fc(H*W*C -> hidden) ReLU fc(hidden -> classes).           default 28x28x1, hidden 128
 *   LENET    conv k x k (no padding, c1) ReLU maxpool2  conv k x k (c2) ReLU maxpool2
 *            fc(fc) ReLU fc(classes).                                   default 28x28x1, 20/50, k 5, fc 500
 *   ALLCNN_C 3x3 convs ca, ca, ca (stride 2), cb, cb, cb (stride 2), cb, all padding 1;
 *            1x1 convs cb, classes; ReLU after every conv but the last; global average pool.
 *                                                                       default 32x32x3, 96/192
 *   WRN      conv3x3(C -> base); three groups of nb blocks, widths base*widen*{1,2,4}, first
 *            block of groups 2 and 3 has stride 2; block = BN ReLU conv3x3 BN ReLU conv3x3 plus
 *            the block input, or plus a strided 1x1 conv of the first BN-ReLU output when the
 *            shape changes; BN ReLU, global average pool, fc.  No conv bias.  BN: batch statistics
 *            per replica (biased variance), eps 1e-5, running statistics with momentum 0.1 and
 *            unbiased variance.                                         default 32x32x3, 16/4/2 (WRN-16-4)
 *   LENET with lenet_bn = 1 (Section 4.2 lists batch-norm for LeNet): batch-norm follows both
 *            convolutions and fc1, before the ReLU; segments bn1, bn2, bn3 follow conv1, conv2, fc1.
 * Dropout (Section 4: 0.25 LeNet, 0.3 / 0.4 wide residual networks, 0.5 All-CNN; `dropout` = 0 switches
 * it off): sites are LENET after each pooling and after fc's ReLU, ALLCNN_C after its two stride-2
 * convolutions, WRN between the two convolutions of every block; numbered in execution order.
 * Element i of site s of replica a at inner step k (the value of k before the step) is kept iff
 *   (mix(mix(i ^ key) + key) >> 8) >= floor(dropout * 2^24),
 *   key = mix(mix(seed + 0x9E3779B9*k) ^ (a*0x85EBCA6B + s*0xC2B2AE35 + 1)),   all modulo 2^32,
 *   mix(x): x ^= x >> 16; x *= 0x7FEB352D; x ^= x >> 15; x *= 0x846CA68B; x ^= x >> 16,
 * kept elements are multiplied by 1 / (1 - dropout); parle_eval applies no dropout.
 * The multipliers are public-domain integer-hash constants, not the paper's: 0x7FEB352D / 0x846CA68B
 * with shifts 16-15-16 are the "lowbias32" finaliser found by C. Wellons' hash-prospector search,
 * 0x9E3779B9 is 2^32 / golden ratio (Knuth's multiplicative hashing), 0x85EBCA6B / 0xC2B2AE35 are the
 * two multipliers of MurmurHash3's 32-bit finaliser (A. Appleby); here the last three only decorrelate
 * the counters that enter the key.
 * Loss: mean over the replica's mini-batch of the softmax cross-entropy (Section 1.1).
 * ReLU'(0) = 0.  maxpool2 = 2x2 window, stride 2, floor; gradient to the first maximum in
 * row-major window order.
 */
typedef struct {
  int32_t model;         /* parle_model */
  int32_t n_replicas;    /* n >= 1 */
  int32_t batch;         /* mini-batch per replica (ignored for FLAT) */
  int32_t L;             /* inner steps per outer step (Section 3.1: 25); advisory, see parle_outer_step */
  int32_t compute_bf16;  /* 0: fp32 activations and MFMA; 1: bf16 activations/weights in the
                            contractions, fp32 accumulation, fp32 master state */
  int32_t in_h, in_w, in_c, n_classes; /* 0 = model default */
  int32_t arch[4];       /* model-specific sizes listed at parle_model; 0 = default */
  int64_t n_params;      /* FLAT only: elements per replica; ignored otherwise */
  float eta_inner;       /* eta'  of (8a) */
  float eta_outer;       /* eta   of (8c) */
  float momentum;        /* Nesterov momentum of the y^a and x^a updates (remark in Section 3): 0.9 */
  float alpha;           /* averaging constant of (8b): 0.75 */
  float weight_decay;    /* coefficient of the 0.5*||y||^2 regulariser inside f (Section 1.1) */
  float gamma0, rho0;    /* initial multipliers g, r (paper: 1/100 and 1) */
  float gamma_max, rho_max; /* caps on g, r (paper clips gamma at 1, rho at 0.1: caps 1 and 10) */
  int64_t scoping_B;     /* B of rule (9), mini-batches in the data set; 0 = g, r stay constant */
  int32_t xa_mode;       /* coefficient on (x^a - z^a) in (8c): 0 = g (unscaled local-entropy
                            gradient of the scoping remark), 1 = 1 (equation as printed) */
  int32_t xref_mode;     /* 0 = (8c) uses the mean of the current replicas; 1 = uses the stored
                            reference, which is then refreshed from the replicas before the move */
  int32_t reset_flags;   /* at the outer step: bit 0 z^a <- x^a, bit 1 momentum of y^a <- 0 */
  int32_t fuse_outer;    /* 0 = replica-mean kernel then outer-update kernel; 1 = one kernel */
  int32_t algorithm;     /* parle_algorithm */
  int32_t graph_block;   /* 1 = parle_inner_block replays a captured HIP graph (see there); 0 = it enqueues
                            the steps one by one */
  float dropout;         /* dropout probability in [0, 1) at the sites listed above; 0 = off */
  int32_t lenet_bn;      /* LENET: 1 = batch-norm after conv1, conv2 and fc1 */
  int64_t dropout_seed;  /* low 32 bits seed the keep-masks */
} parle_config;

typedef struct {
  int64_t n_params;        /* parameters per replica */
  int64_t n_pad;           /* row stride in elements: n_params rounded up to a multiple of 1024 */
  int64_t state_bytes;     /* bytes of ONE [n, n_pad] fp32 tensor (x, y, z, vy, vx, grad each) */
  int64_t shadow_bytes;    /* bytes of the [n, n_pad] bf16 copy of y; 0 when compute_bf16 == 0 */
  int64_t bn_bytes;        /* bytes of the batch-norm running statistics; 0 without BN */
  int64_t workspace_bytes; /* bytes of scratch the kernels need (activations, partial sums) */
  int32_t n_segments;      /* entries parle_query_layout can return */
  int32_t image_elems;     /* H*W*C of one input image; 0 for FLAT */
  int64_t forward_flops_per_image; /* 2*M*N*K summed over the contractions of one forward pass, per image */
} parle_sizes;

typedef enum { PARLE_SEG_WEIGHT = 0, PARLE_SEG_BIAS = 1, PARLE_SEG_BN_GAMMA = 2, PARLE_SEG_BN_BETA = 3 } parle_seg_kind;

typedef struct {
  char name[32];      /* e.g. "conv1.w", "g2b1.bn1.g" */
  int64_t offset;     /* first element inside a replica row */
  int64_t size;       /* elements */
  int32_t kind;       /* parle_seg_kind */
  int32_t shape[4];   /* [Cout,kh,kw,Cin], [out,in,0,0] or [C,0,0,0] */
  int32_t fan_in;     /* inputs feeding one output unit */
} parle_segment;

typedef struct {            /* DEVICE pointers, caller-owned, each 256-byte aligned */
  float *x;                 /* [n, n_pad] replicas x^a; the caller fills it before parle_init */
  float *y;                 /* [n, n_pad] inner iterates y^a */
  float *z;                 /* [n, n_pad] running averages z^a */
  float *vy;                /* [n, n_pad] momentum of y^a */
  float *vx;                /* [n, n_pad] momentum of x^a */
  float *grad;              /* [n, n_pad] grad f(y^a); written by the backward kernels, or by the caller (FLAT) */
  float *x_ref;             /* [n_pad] reference x */
  void *y_bf16;             /* [n, n_pad] bf16 copy of y, or NULL when compute_bf16 == 0 */
  void *bn_stats;           /* bn_bytes: per replica, per BN layer in order, mean[C] then var[C] (fp32); or NULL */
  void *workspace;          /* workspace_bytes of scratch; contents are undefined between calls */
} parle_buffers;

/* Sizes implied by a configuration.  Pure host code; works without a GPU. */
parle_status parle_query_sizes(const parle_config *cfg, parle_sizes *out);

/* Segment `index` (0 <= index < n_segments) of the packing of one replica row.  Pure host code. */
parle_status parle_query_layout(const parle_config *cfg, int32_t index, parle_segment *out);

/*
 * Start of training (Section 3): takes x (all n rows filled by the caller, padding zero) and
 * enqueues y <- x, z <- x, vy <- 0, vx <- 0, grad <- 0, x_ref <- replica mean (8d), bf16 copy,
 * BN running statistics <- (0, 1); sets k = 0, g = gamma0, r = rho0.
 * `hip_stream` is a hipStream_t (NULL = the default stream).  *out is freed by parle_destroy.
 */
parle_status parle_init(const parle_config *cfg, const parle_buffers *buf, void *hip_stream, parle_ctx **out);

/*
 * One inner step for all replicas: forward, loss, backward into buffers.grad, then
 *   d = grad + weight_decay*y + g*(y - x);  vy <- mu*vy + d;  y <- y - eta_inner*(d + mu*vy)   (8a)
 *   z <- alpha*z + (1 - alpha)*y                                                               (8b)
 * images_dev: [n, batch, H, W, C] fp32, labels_dev: [n, batch] int32 in [0, classes);
 * loss_dev: [n] fp32 mean loss of each replica at y before the step, or NULL.
 * FLAT: images_dev and labels_dev must be NULL; only the update runs on the caller's grad.
 */
parle_status parle_inner_step(parle_ctx *ctx, const float *images_dev, const int32_t *labels_dev, float *loss_dev);
/*
 * With algorithm = PARLE_ALG_ELASTIC the same call is one Elastic-SGD step (Section 2.2): forward,
 * loss, backward at the replicas, then for every replica and the reference, all from the old values,
 *   d = grad + weight_decay*x^a + r*(x^a - x);  v <- mu*v + d;  x^a <- x^a - eta_inner*(d + mu*v)
 *   x <- x - eta_outer*(x - (1/n) sum_a x^a)
 */

/*
 * `steps` consecutive inner steps, equal in effect to calling parle_inner_step on
 * images_dev + s*n*batch*H*W*C, labels_dev + s*n*batch, loss_dev + s*n for s = 0 .. steps-1
 * (the latency-bound small networks spend their time in launches, Section 4.1's LeNet being the case
 * in the paper).  With graph_block = 1 the second call with the same four arguments records the
 * launches into a HIP graph and later calls with those arguments replay it; other arguments run
 * step by step and replace the remembered ones.  The graph runs on a stream of the library's own,
 * ordered after and before the init stream with events, so the caller sees the usual stream order.
 * The coupling multipliers are read from device memory inside the graph: scoping needs no re-capture.
 * Not for FLAT (the caller writes the gradient between steps).  1 <= steps <= 4096.
 */
parle_status parle_inner_block(parle_ctx *ctx, const float *images_dev, const int32_t *labels_dev, int32_t steps,
                               float *loss_dev);

/*
 * The outer step, meant to follow every L inner steps (any count >= 1 is accepted, else ESTATE):
 *   x_ref <- (1/n) sum_a x^a                                                   (8d), eta'' = rho/n
 *   d = c_z*(x^a - z^a) + r*(x^a - x_ref);  vx <- mu*vx + d;  x^a <- x^a - eta_outer*(d + mu*vx)   (8c)
 *   y^a <- x^a (and z^a, vy per reset_flags), bf16 copy refreshed
 *   g <- min(g / (1 - 1/(2B)), gamma_max), r likewise                         rule (9)
 * With algorithm = PARLE_ALG_ELASTIC no kernel runs: only r advances by rule (9).
 */
parle_status parle_outer_step(parle_ctx *ctx);

/*
 * Forward only, at the reference (which = -1; BN uses running statistics averaged over the
 * replicas) or at replica `which`'s x^a (buffers.x; buffers.y for Elastic-SGD).  images_dev [count, H, W, C], labels_dev [count],
 * 1 <= count <= n*batch.  Writes to HOST: mean loss, number of misclassified samples, and (if
 * not NULL) spread = sum_a ||x^a - x_ref||^2.  Blocks until the stream is idle.
 * FLAT: images/labels must be NULL, count 0; only spread is produced.
 * PARLE_ENONFINITE if the mean loss is NaN or infinite (the outputs are written all the same, the context stays
 * usable).  It sees what reaches the logits: a NaN in front of a ReLU is turned into 0 by it (`v > 0 ? v : 0`)
 * and is not reported.
 */
parle_status parle_eval(parle_ctx *ctx, int32_t which, const float *images_dev, const int32_t *labels_dev,
                        int32_t count, float *loss_host, int32_t *n_err_host, float *spread_host);

/* Scalars a caller needs to checkpoint / resume: inner steps taken, completed outer steps, g, r. */
parle_status parle_get_state(const parle_ctx *ctx, int64_t *k, int64_t *outer_done, float *g, float *r);
parle_status parle_set_state(parle_ctx *ctx, int64_t k, int64_t outer_done, float g, float r);

/* Text of the last error on this context (or of the last failed init when ctx == NULL). */
const char *parle_last_error(const parle_ctx *ctx);

/* Frees the host context.  Never touches the caller's device buffers.  NULL is allowed. */
void parle_destroy(parle_ctx *ctx);

/* ------------------------------------------------------------------------------------------
 * Single-kernel entry points (the steps above, one launch each, on arbitrary caller state).
 * All pointers are DEVICE pointers, 16-byte aligned; n_pad must be a multiple of 4 and
 * n*n_pad < 2^40.  Enqueued on `hip_stream`; asynchronous.
 * ------------------------------------------------------------------------------------------ */

/* (8a) + Nesterov + (8b) on [n, n_pad]; y_bf16 may be NULL. */
parle_status parle_k_inner_update(void *hip_stream, int32_t n, int64_t n_pad, const float *grad, const float *x,
                                  float *y, float *vy, float *z, void *y_bf16, float eta_inner, float momentum,
                                  float alpha, float weight_decay, float g);

/* Elastic-SGD (Section 2.2), both updates in one launch, all from the old values:
 *   d = grad + weight_decay*xa + r*(xa - x_ref);  v <- momentum*v + d;  xa <- xa - eta*(d + momentum*v)
 *   x_ref <- x_ref - eta_ref*(x_ref - mean_a xa)
 * xa, v, grad: [n, n_pad]; x_ref: [n_pad]; xa_bf16 may be NULL. */
parle_status parle_k_elastic_step(void *hip_stream, int32_t n, int64_t n_pad, const float *grad, float *xa, float *v,
                                  float *x_ref, void *xa_bf16, float eta, float eta_ref, float momentum,
                                  float weight_decay, float r);

/* (8d) with eta'' = rho/n: x_ref[i] = (sum_{a=0..n-1} x[a][i]) / n, summed in replica order. */
parle_status parle_k_replica_mean(void *hip_stream, int32_t n, int64_t n_pad, const float *x, float *x_ref);

/* (8c) + Nesterov + reset.  c_z is the coefficient on (x - z).  fuse_mean = 1 computes the
 * replica mean inside the kernel and writes it to x_ref; lagged = 1 applies xref_mode 1. */
parle_status parle_k_outer_update(void *hip_stream, int32_t n, int64_t n_pad, float *x, float *z, float *vx,
                                  float *y, float *vy, float *x_ref, void *y_bf16, float eta_outer, float momentum,
                                  float c_z, float r, int32_t reset_flags, int32_t fuse_mean, int32_t lagged);

/* sum_a ||x^a - x_ref||^2 -> out_dev[0] (fp32).  partial_dev: scratch of >= 4096 doubles. */
parle_status parle_k_spread(void *hip_stream, int32_t n, int64_t n_pad, const float *x, const float *x_ref,
                            double *partial_dev, float *out_dev);

/* parle_k_spread for callers that cannot allocate device memory or pass a scratch buffer along: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same result, same
 * kernels; the per-workgroup partial sums live in a 32 KiB array that is part of the library's device
 * image (one copy per GPU, held until the process ends), and the call allocates and frees nothing.
 * x, x_ref, out_dev as for parle_k_spread (device pointers, 16-byte aligned, caller-owned; out_dev[0]
 * receives the fp32 sum).  n * n_pad <= PARLE_SPREAD_STATIC_MAX_ELEMS, else PARLE_ESIZE; EINVAL / EALIGN /
 * EHIP as usual, with a text behind parle_last_error(NULL).  Every call on a GPU uses that GPU's one
 * array: calls that overlap on one GPU (different streams, different threads) race on it and must be
 * ordered by the caller; calls on one stream are safe.  Nothing in the array needs clearing between
 * calls: the second kernel reads only the slots the first kernel of the same call wrote. */
#define PARLE_SPREAD_STATIC_MAX_ELEMS (1LL << 34)
parle_status parle_k_spread_static(void *hip_stream, int32_t n, int64_t n_pad, const float *x, const float *x_ref,
                                   float *out_dev);

/* Measurement aid, not a step of the method: `reads` arrays of `count` floats are read from src_dev
 * (laid out one after the other) and `writes` arrays of `count` floats written to dst_dev, with the
 * access shape of the update kernels (16 bytes per lane, non-temporal) and no arithmetic that matters.
 * The rate it reaches is what the memory system gives that mix; (reads, writes) must be (1,0), (0,1),
 * (1,1) or (5,3), the last being the mix of the fused inner update.  count % 4 == 0; dst_dev holds
 * max(writes, 1) * count floats (a read-only run writes nothing for finite inputs); EINVAL otherwise. */
parle_status parle_k_stream_reference(void *hip_stream, int32_t reads, int32_t writes, int64_t count,
                                      const float *src_dev, float *dst_dev);

/* ------------------------------------------------------------------------------------------
 * The replica-grouped convolution kernels behind grad f(y^a) of (8a), one launch each.
 * Tensors are DEVICE pointers, 16-byte aligned, channels-last, one block per replica:
 *   x  [n][batch, h, w, cin]      w  [n][cout, k, k, cin]      y, dy [n][batch, ho, wo, cout]
 * with ho = (h + 2 pad - k)/stride + 1.  dtype 0: fp32 tensors; dtype 1: bf16 tensors (raw 16-bit),
 * products accumulated in fp32 on the MFMA units.  stride is 1 or 2.  A fully connected layer is
 * h = w = k = 1.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t dtype, n, batch, h, w, cin, cout, k, stride, pad;
} parle_conv_desc;

/* y = [relu]( conv(x, w) + bias + resid ); bias [n][cout] fp32 or NULL; resid like y or NULL. */
parle_status parle_k_conv_forward(void *hip_stream, const parle_conv_desc *desc, const void *x, const void *w,
                                  const float *bias, const void *resid, int32_t relu, void *y);

/* The same forward convolution (no bias, no ReLU: the form in front of a batch-norm of the residual
 * networks) that also leaves, for the batch-norm statistics of its output, column sums taken in its
 * epilogue: partial [n][S][2][cout] doubles, row s of replica a holding the sums over a group of
 * output rows of y (as stored, i.e. after rounding to dtype) and of their squares; summing the S rows
 * gives the sums over all batch*ho*wo rows.  S is written to *splits_host (HOST); S = 0 means the kernel
 * that runs this layer takes no sums (then `partial` is untouched and the caller reduces y itself).
 * `capacity`: rows per replica `partial` has room for (S never exceeds it). */
parle_status parle_k_conv_forward_colsums(void *hip_stream, const parle_conv_desc *desc, const void *x, const void *w,
                                          const void *resid, void *y, double *partial, int32_t capacity,
                                          int32_t *splits_host);
/* dx (+)= conv^T(dy, w), multiplied by (relu_mask > 0) when relu_mask (like x) is given.
 * wt_scratch: n*cout*k*k*cin elements of the tensor dtype (receives the transposed weights). */
parle_status parle_k_conv_backward_data(void *hip_stream, const parle_conv_desc *desc, const void *dy, const void *w,
                                        const void *relu_mask, int32_t accumulate, void *wt_scratch, void *dx);
/* dw [n][cout, k, k, cin] fp32 = sum over batch and positions of dy (x) x.  The sum is split over
 * workgroups and reduced in a fixed order; scratch must hold parle_k_conv_scratch_bytes(desc). */
parle_status parle_k_conv_backward_weight(void *hip_stream, const parle_conv_desc *desc, const void *dy, const void *x,
                                          float *scratch, int64_t scratch_bytes, float *dw);
/* The same weight gradient with the layer's bias gradient (Section 1.1's loss differentiated with
 * respect to a per-channel offset of y: the sum of dy over batch and positions) taken along by the
 * kernels that read all of dy anyway: dwb [n][cout*k*k*cin + cout] fp32, each replica's bias gradient
 * behind its weight gradient, as the two segments lie in a parameter row.  *took_bias_host (HOST) = 1
 * when the kernel that runs this layer wrote the cout bias values, 0 when it left them untouched (the
 * caller then sums dy itself, parle_k_bias_grad).  Scratch as above. */
parle_status parle_k_conv_backward_weight_bias(void *hip_stream, const parle_conv_desc *desc, const void *dy,
                                               const void *x, float *scratch, int64_t scratch_bytes, float *dwb,
                                               int32_t *took_bias_host);
int64_t parle_k_conv_scratch_bytes(const parle_conv_desc *desc); /* -1 on a bad descriptor; covers both forms */

/* ------------------------------------------------------------------------------------------
 * The memory-bound layer kernels of the same forward / backward pass (Section 1.1's loss; the
 * batch-norm, dropout and pooling layers of the networks of Section 4), one layer each.
 * Tensors are DEVICE pointers, 16-byte aligned, channels-last, one block per replica:
 *   [n][batch, h, w, c] in the activation format (dtype 0: fp32, 1: bf16 raw 16-bit; results are
 *   computed in fp32 and rounded to nearest even once, on the store).
 * Per-channel parameters and results are fp32 [n][c].  `scratch` holds the partial sums of the
 * column reductions: parle_k_layer_scratch_bytes(desc) bytes (-1 on a bad descriptor), ESIZE if less.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t dtype, n, batch, h, w, c;
} parle_act_desc;
int64_t parle_k_layer_scratch_bytes(const parle_act_desc *desc);

/* Training-mode batch-norm + ReLU: per replica and channel, mean and biased variance over the
 * batch*h*w rows; out = max(0, gamma*(x - mean)/sqrt(var + 1e-5) + beta).  saved [n][2][c] receives
 * mean and 1/sqrt(var + eps); running [n][2][c] (mean, variance; may be NULL) is updated with momentum 0.1
 * and the unbiased variance. */
parle_status parle_k_bn_forward(void *hip_stream, const parle_act_desc *desc, const void *x, const float *gamma,
                                const float *beta, void *scratch, int64_t scratch_bytes, float *saved, float *running,
                                void *out);
/* Its backward: with xhat = (x - mean)*rstd and d = dout where gamma*xhat + beta > 0, else 0:
 *   dbeta = sum d, dgamma = sum d*xhat, dx = gamma*rstd*(d - dbeta/M - xhat*dgamma/M) (+ add, like x, or NULL).
 * sums [n][2][c] is a work buffer (the two sums in fp32). */
parle_status parle_k_bn_backward(void *hip_stream, const parle_act_desc *desc, const void *x, const void *dout,
                                 const float *gamma, const float *beta, const float *saved, const void *add,
                                 void *scratch, int64_t scratch_bytes, float *sums, float *dgamma, float *dbeta, void *dx);
/* 2x2 max-pool, stride 2, floor: in [n][batch,h,w,c] -> out [n][batch,h/2,w/2,c].  Backward: dout goes to the
 * first maximum of each window in row-major order (times (in > 0) when relu_mask != 0), zero elsewhere. */
parle_status parle_k_maxpool_forward(void *hip_stream, const parle_act_desc *desc, const void *in, void *out);
parle_status parle_k_maxpool_backward(void *hip_stream, const parle_act_desc *desc, const void *in, const void *dout,
                                      int32_t relu_mask, void *din);
/* Global average pool over h*w: out [n][batch, c] (fp32 when out_f32 != 0, else the activation format);
 * backward: din = dout / (h*w) at every position. */
parle_status parle_k_gap_forward(void *hip_stream, const parle_act_desc *desc, int32_t out_f32, const void *in, void *out);
parle_status parle_k_gap_backward(void *hip_stream, const parle_act_desc *desc, const void *dout, void *din);
/* Dropout with the keep-mask defined at parle_config (site `site`, rate p, inner step read from step_dev[0]):
 * out = keep ? in / (1 - p) : 0, additionally zero where relu_src <= 0 when relu_src (like in) is given.
 * The same call applied to a gradient is the backward pass. */
parle_status parle_k_dropout(void *hip_stream, const parle_act_desc *desc, const void *in, const void *relu_src,
                             uint32_t seed, const int64_t *step_dev, int32_t site, float p, void *out);
/* grad [n][c] = sum over the batch*h*w rows of dy (the bias gradient of a layer). */
parle_status parle_k_bias_grad(void *hip_stream, const parle_act_desc *desc, const void *dy, void *scratch,
                               int64_t scratch_bytes, float *grad);
/* Mean softmax cross-entropy of each replica's batch: logits fp32 [n][batch, classes], labels [n][batch];
 * loss [n] (may be NULL); dlogits (activation format) = (softmax - onehot) / batch. */
parle_status parle_k_softmax_xent(void *hip_stream, int32_t dtype, int32_t n, int32_t batch, int32_t classes,
                                  const float *logits, const int32_t *labels, float *loss, void *dlogits);

/* The classifier's last fully connected layer, the loss above and the layer's input gradient as ONE kernel (what a
 * training step of the networks that end in such a layer runs): feat [n][batch, features], w [n][classes, features]
 * (activation format), bias [n][classes] fp32 or NULL, 1 <= classes <= 16, (classes + 8) * features <= 16384.
 *   logits = feat w^T + bias;  dlogits [n][batch, classes] = (softmax - onehot) / batch, stored in the activation
 *   format;  dfeat [n][batch, features] = dlogits (as stored) x w, zero where relu_mask != 0 and feat <= 0.
 * loss_img [n][batch] fp32 receives the per-image cross-entropies, loss [n] (may be NULL) their means. */
parle_status parle_k_fc_head(void *hip_stream, int32_t dtype, int32_t n, int32_t batch, int32_t features,
                             int32_t classes, const void *feat, const void *w, const float *bias, const int32_t *labels,
                             int32_t relu_mask, float *loss_img, float *loss, void *dlogits, void *dfeat);

/* The same for a network that ends in a global average pool over class maps (All-CNN-C): feat [n][batch, h, w, c]
 * with c <= 16 classes; logits = mean over the h*w pixels; dlogits [n][batch, c] as above;
 * dfeat [n][batch, h, w, c] = dlogits / (h*w) at every pixel; loss_img, loss as above. */
parle_status parle_k_gap_head(void *hip_stream, const parle_act_desc *desc, const void *feat, const int32_t *labels,
                              float *loss_img, float *loss, void *dlogits, void *dfeat);

#ifdef __cplusplus
}
#endif
#endif /* PARLE_H */
