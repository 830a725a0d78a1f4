// Replica-grouped implicit-GEMM convolutions on MFMA (gfx950): forward / backward-data share one
// gather kernel, backward-weight is a split-K kernel.  Fully connected layers are 1x1 convolutions
// on a 1x1 image.  blockIdx.z walks the replicas (and the K-splits of backward-weight).
#pragma once
#include "common.h"

// n / d for 0 <= n < 2^31 by multiply-high (no integer division on the device).
struct FastDiv {
  uint32_t d, magic, shift;
};
inline FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t s = 0;
  while ((1u << s) < d) ++s;
  f.shift = 31 + s;
  f.magic = (uint32_t)((((uint64_t)1 << (31 + s)) + d - 1) / d);
  return f;
}

// Rows m = (b, p, q) over a P x Q grid; contraction index k = (r, s, c) over an R x S window and
// Cc channels of a channels-last tensor [*, Hin, Win, Cc].  Tap position along h:
//   t = p*sp + off + r*sr;  valid iff t >= 0, t divisible by 2^dshift, (t >> dshift) < Hin
// forward conv:   sp = stride, off = -pad, sr = +1, dshift = 0   (gathers the layer input)
// backward data:  sp = 1, off = +pad, sr = -1, dshift = log2(stride) (gathers the output gradient)
struct ConvGeom {
  int Hin, Win, Cc;
  int P, Q;
  int R, S;
  int sp, off, sr, dshift;
  int M, N, K;  // per replica: rows, output columns, contraction length (K = R*S*Cc)
  FastDiv dPQ, dQ, dCc, dS;
  // Row order inside an image.  0: natural (p, q).  Otherwise log2 P and log2 Q (both >= 1): the rows
  // of an image are grouped by the parity class (p % 2, q % 2), class-major, so that the rows of a
  // tile share the taps that a stride-2 backward-data gather can reach.  Only kernels that say so
  // honour it; the launchers set it, not the callers.
  int plp, plq;
  // With plp, plq >= 4 and pblk != 0 the order inside an image is instead: block of 16 x 16 pixels
  // (row-major over the blocks), parity class, position (i, j) of the 8 x 8 grid inside the block, i.e.
  // pixel (16*bi + 2*i + class/2, 16*bj + 2*j + class%2): a 256-row tile is one block, 64 rows per class.
  int pblk;
  // Backward-weight only: wavefronts a launch of the nine-tap kernel should put in flight (0 = one per SIMD of
  // the chip); the contraction is split over workgroups accordingly.
  int leaf_waves;
};

struct GemmIO {
  const void *in;    // gathered tensor
  long long in_rs;   // replica stride, elements
  const void *w;     // [N][K] row-major
  long long w_rs;
  void *out;         // [M][ldc]
  long long out_rs;
  int ldc;
  const float *bias;  // [N] fp32 or NULL
  long long bias_rs;
  const void *resid;  // [M][ldc], added before the ReLU, or NULL
  long long resid_rs;
  const void *mask;   // [M][ldc]: result multiplied by (mask > 0), or NULL
  long long mask_rs;
  int relu, accumulate;
  int vecA, vecB;     // 16-byte loads allowed for the gathered operand / the weight matrix
  long long in_bytes; // bytes of one replica's gathered tensor (range of the buffer loads)
  // The gathered tensor lies in memory as fp32 although the layer computes in bf16 (the caller's images in front of a
  // first layer): values are rounded to bf16 as they are gathered.  Only the small-window kernel takes it;
  // launch_igemm fails for a layer that kernel does not run.
  int in_f32;
  // Column sums of the stored output and of its squares, per workgroup of pixel rows, for the batch-norm that
  // follows: [replica][S][2][ldc] doubles, or NULL.  Only launch_igemm's callers that ask for the split count
  // set it; kernels that do not produce the sums ignore it and launch_igemm reports S = 0.
  double *stat;
  int stat_capacity;  // partial rows per replica the buffer has room for
};

struct WgradIO {
  const void *dy;  // [M][N] output gradient
  long long dy_rs;
  const void *x;   // layer input, gathered with the forward geometry
  long long x_rs;
  float *out;      // [N][K] fp32 per (replica, split)
  long long out_rs, split_stride;
  int splits, chunk;  // K-splits over M and rows of M per split (multiple of 32)
  int pairA, pairB;   // packed loads allowed for dy / x
  // Kernels that can (see wgrad_takes_bias) also write the layer's bias gradient, the column sums of dy, behind the
  // N*K weight-gradient values of `out`: N more floats per (replica, split).  In a parameter row the bias segment
  // follows the weight segment, so the one reduction over the splits, or the direct write, covers both.
  int with_bias;
  int x_f32;  // x lies in memory as fp32 (see GemmIO::in_f32); only the small-window bf16 kernel takes it
};

// A convolution layer as the kernels see it: [B, H, W, Cin] -> [B, Ho, Wo, Cout], R x R window.
struct ConvShape {
  int B, H, W, Cin, Cout, R, stride, pad;
  int Ho() const { return (H + 2 * pad - R) / stride + 1; }
  int Wo() const { return (W + 2 * pad - R) / stride + 1; }
};
inline ConvGeom conv_fwd_geom(const ConvShape &c) {
  ConvGeom g{};
  g.Hin = c.H, g.Win = c.W, g.Cc = c.Cin;
  g.P = c.Ho(), g.Q = c.Wo(), g.R = c.R, g.S = c.R;
  g.sp = c.stride, g.off = -c.pad, g.sr = 1, g.dshift = 0;
  g.M = c.B * g.P * g.Q, g.N = c.Cout, g.K = c.R * c.R * c.Cin;
  g.dPQ = make_fastdiv(g.P * g.Q), g.dQ = make_fastdiv(g.Q), g.dCc = make_fastdiv(g.Cc), g.dS = make_fastdiv(g.S);
  return g;
}
// Gradient w.r.t. the input: gathers the output gradient; stride must be 1 or 2.
inline ConvGeom conv_bwd_geom(const ConvShape &c) {
  ConvGeom g{};
  g.Hin = c.Ho(), g.Win = c.Wo(), g.Cc = c.Cout;
  g.P = c.H, g.Q = c.W, g.R = c.R, g.S = c.R;
  g.sp = 1, g.off = c.pad, g.sr = -1, g.dshift = c.stride == 2 ? 1 : 0;
  g.M = c.B * c.H * c.W, g.N = c.Cin, g.K = c.R * c.R * c.Cout;
  g.dPQ = make_fastdiv(g.P * g.Q), g.dQ = make_fastdiv(g.Q), g.dCc = make_fastdiv(g.Cc), g.dS = make_fastdiv(g.S);
  return g;
}

// dtype: 0 = fp32 (v_mfma_f32_32x32x2_f32), 1 = bf16 (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
// `stat_splits`: with io.stat set, receives the number S of partial rows of column sums the kernel writes
// (0: the kernel that runs this layer does not produce them; the caller takes them in a pass of its own).
hipError_t launch_igemm(hipStream_t st, int dtype, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io,
                        int *stat_splits = nullptr);
hipError_t launch_wgrad(hipStream_t st, int dtype, int replicas, const ConvGeom &g, const WgradIO &io);
// Vector fast paths (igemm_fast.hip); launch_igemm / launch_wgrad pick them when applicable.
bool igemm_fast_applicable(int dtype, const ConvGeom &g, const GemmIO &io);
hipError_t launch_igemm_fast(hipStream_t st, int dtype, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io);
int igemm_fast_stat_splits(int dtype, bool out_f32, const ConvGeom &g, const GemmIO &io);
// Stride-1 'same' convolutions with the input patch staged once in LDS (igemm_halo.hip).
bool conv_halo_applicable(int dtype, const ConvGeom &g, const GemmIO &io, bool out_f32);
hipError_t launch_conv_halo(hipStream_t st, int replicas, const ConvGeom &g, const GemmIO &io);
int conv_halo_stat_splits(const ConvGeom &g, int replicas);
// fp32 backward-data of a stride-1 layer with few input channels under a wide window, the per-tap products of one
// image held in LDS (igemm_dgrad_win.hip).  w: the layer's weights as they lie, [Cout][R][R][Cin].
// ... and its backward-weight pass with the window gather in LDS (splits over images; partial sums per split).
bool wgrad_window_applicable(int dtype, const ConvGeom &g);
int wgrad_window_plan(int replicas, const ConvGeom &g, int *chunk_out);
hipError_t launch_wgrad_window(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io);
bool dgrad_window_applicable(int dtype, int B, int H, int W, int Cin, int Cout, int R, int stride, int pad);
hipError_t launch_dgrad_window(hipStream_t st, int n, int B, int H, int W, int Cin, int Cout, int R, int pad,
                               const float *dy, long long dy_rs, const float *w, long long w_rs,
                               const float *mask, long long mask_rs, int accumulate, float *dx, long long dx_rs);
bool wgrad_fast_applicable(int dtype, const ConvGeom &g);
void wgrad_fast_tile(const ConvGeom &g, int *bm, int *bn);
hipError_t launch_wgrad_fast(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io);
// Layers whose whole contraction fits one tile, K = R*S*Cin <= 32 (igemm_smallk.hip).
bool conv_smallk_applicable(int dtype, const ConvGeom &g, const GemmIO &io);
hipError_t launch_conv_smallk(hipStream_t st, int dtype, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io);
int conv_smallk_stat_splits(const ConvGeom &g, bool out_f32);
bool wgrad_smallk_applicable(int dtype, const ConvGeom &g);
hipError_t launch_wgrad_smallk(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io);
// Stride-1 'same' 3x3 backward-weight with the patch staged in LDS and nine taps per wavefront (igemm_wgrad9.hip).
bool wgrad9_applicable(int dtype, const ConvGeom &g);
int wgrad9_plan(int replicas, const ConvGeom &g, int *chunk_out);
hipError_t launch_wgrad9(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io);
// Plain products with few output tiles: the contraction split over the wavefronts of a workgroup (igemm_ksplit.hip).
bool gemm_ksplit_applicable(int dtype, int replicas, const ConvGeom &g, const GemmIO &io);
hipError_t launch_gemm_ksplit(hipStream_t st, int dtype, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io);
// fp32 backward-weight with at most 32 output channels and a window of at most 32 values (igemm_ksplit.hip).
bool wgrad_small_f32_applicable(int dtype, const ConvGeom &g);
// True when launch_wgrad would run a kernel that honours WgradIO::with_bias for this layer and these operands
// (io.dy, io.pairA, io.pairB set): the small-window kernels when the window leaves one of their 32 contraction
// columns unused, the stride-1 3x3 kernel, the transpose-read kernel and the generic fp32 kernel.
bool wgrad_takes_bias(int dtype, const ConvGeom &g, const WgradIO &io);
hipError_t launch_wgrad_small_f32(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io);
// Backward-data of stride-2 3x3 pad-1 layers, four parity classes per workgroup (igemm_dgrad2.hip).
bool dgrad_s2_applicable(int dtype, const ConvGeom &g, const GemmIO &io, bool out_f32);
hipError_t launch_dgrad_s2(hipStream_t st, int replicas, const ConvGeom &g, const GemmIO &io);
// Rows of M per split so that the launch has enough workgroups; returns the split count.
int wgrad_plan(int dtype, int replicas, const ConvGeom &g, int *chunk_out);
