// Backward-data of a stride-1 convolution with few input channels under a wide window, fp32 (LeNet's second
// convolution: 20 channels, 5 x 5 taps, 8 x 8 outputs), one image per workgroup, in ONE kernel:
//
//   col[m][(r, s, ci)] = sum_n dy[m][n] * w[n][r][s][ci]          a plain matrix product over the output channels
//   dx[h][w][ci]       = sum_{r, s} col[(h + pad - r, w + pad - s)][(r, s, ci)]
//
// As a direct implicit GEMM the pass has Cin = 20 of 32 MFMA columns in use and a contraction of R*S*Cout; as two
// kernels (the product, then the gather over the window) every entry of col travels to memory and back, 100 MB
// for the layer above.  Here col of ONE image stays in LDS (P*Q x R*S*Cin floats: 125 KB for that layer): the
// workgroup multiplies its image's dy tile, held in LDS, with the weights read straight from memory into MFMA
// fragments - as they lie, [Cout][R*S*Cin], they are the [K][N] operand, so the 32 lanes of a fragment half read 32
// consecutive floats - parks the product in LDS and gathers from there.  One workgroup per compute unit (LDS),
// eight wavefronts.
#include "igemm_dev.h"

namespace {

using namespace igemm_dev;

constexpr int kWinThreads = 512;
constexpr int kWinMaxPix = 64;    // output pixels of an image: two 32-row MFMA tiles
constexpr int kWinMaxCout = 64;   // contraction length
constexpr int kWinLdsBytes = 160 * 1024;

struct WinGeom {
  int B, H, W, Cin, Cout, R, pad, P, Q;  // dx [B][H][W][Cin], dy [B][P][Q][Cout]
  int NC;                                // R*R*Cin: columns of col
  int KG;                                // contraction groups of 8
  int lda, ldc;                          // LDS row pitches (floats) of the dy tile and of col
  FastDiv dCin, dW, dCout, dCv;          // no integer division on the device
  int vec;                               // Cin % 4 == 0: the gather runs on 16-byte vectors
};

// LDS pitches: the dy tile is read as 16-byte fragments by 32 rows x 2 halves (pitch = 4 mod 32 banks keeps the
// eight 16-byte accesses of a quarter-wavefront apart); col is written 32 consecutive columns at a time and read
// along Cin, so any pitch does
__host__ __device__ inline int win_lda(int Cout) { return (Cout + 7) / 8 * 8 + 4; }

__global__ __launch_bounds__(kWinThreads) void k_dgrad_window(const WinGeom g, const float *__restrict__ dy,
                                                              long long dy_rs, const float *__restrict__ w,
                                                              long long w_rs, const float *__restrict__ mask,
                                                              long long mask_rs, int accumulate, float *__restrict__ dx,
                                                              long long dx_rs) {
  extern __shared__ __attribute__((aligned(16))) float win_lds[];
  float *dyS = win_lds;                       // [64][lda], rows beyond P*Q and columns beyond Cout are zero
  float *colS = win_lds + kWinMaxPix * g.lda;  // [P*Q][ldc]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x, rep = blockIdx.y;
  const int PQ = g.P * g.Q;
  const float *dyp = dy + rep * dy_rs + (long long)b * PQ * g.Cout;
  const float *wp = w + rep * w_rs;

  // dy tile -> LDS (zero padded)
  for (int i = tid; i < kWinMaxPix * g.lda; i += kWinThreads) dyS[i] = 0.f;
  __syncthreads();
  for (int i = tid; i < PQ * g.Cout; i += kWinThreads) {   // the tile is contiguous in memory
    const int m = (int)fdiv((uint32_t)i, g.dCout), k = i - m * g.Cout;
    dyS[m * g.lda + k] = dyp[i];
  }
  __syncthreads();

  // col = dy x w: column tile tn (32 columns of col) per wavefront and trip, both row tiles at once so that a
  // weight fragment serves two MFMAs.  Fragment of half h, element j of group q: contraction index 8q + 4h + j.
  const int r = lane & 31, h = lane >> 5;
  const int n_tiles = (g.NC + 31) / 32;
  for (int tn = wave; tn < n_tiles; tn += kWinThreads / 64) {
    const int col = tn * 32 + r;
    const bool col_ok = col < g.NC;
    const float *wcol = wp + col;   // element (k, col) at wcol[k * NC]
    f16v acc0, acc1;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = 0.f, acc1[v] = 0.f;
    // four groups = 32 contraction values per trip; the fragments of the next trip travel while this one multiplies
    auto load_b = [&](int q0, u4 (&bf)[4]) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int k = 8 * (q0 + u) + 4 * h;
        float t[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) t[j] = (col_ok && k + j < g.Cout) ? wcol[(long long)(k + j) * g.NC] : 0.f;
        bf[u] = u4{__float_as_uint(t[0]), __float_as_uint(t[1]), __float_as_uint(t[2]), __float_as_uint(t[3])};
      }
    };
    u4 cur[4], nxt[4];
    load_b(0, cur);
    for (int q0 = 0; q0 < g.KG; q0 += 4) {
      if (q0 + 4 < g.KG) load_b(q0 + 4, nxt);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (q0 + u < g.KG) {
          const int k = 8 * (q0 + u) + 4 * h;
          const u4 a0 = *(const u4 *)&dyS[r * g.lda + k], a1 = *(const u4 *)&dyS[(32 + r) * g.lda + k];
          mma<float>(a0, cur[u], acc0);
          mma<float>(a1, cur[u], acc1);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
    }
    // accumulator v of a lane: row 8*(v/4) + 4*h + v%4 of its row tile, column r of the column tile
    if (col_ok) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = 8 * (v >> 2) + 4 * h + (v & 3);
        if (m < PQ) colS[m * g.ldc + col] = acc0[v];
        if (32 + m < PQ) colS[(32 + m) * g.ldc + col] = acc1[v];
      }
    }
  }
  __syncthreads();

  // gather over the window, taps in order (the order the two-kernel path adds them in)
  const int total = g.H * g.W * g.Cin;
  const long long img = (long long)b * total;
  const float *mp = mask ? mask + rep * mask_rs + img : nullptr;
  float *op = dx + rep * dx_rs + img;
  if (g.vec) {
    // four consecutive channels per thread: 16-byte LDS reads (pitch and tap offsets are multiples of four floats)
    const int cv = g.Cin >> 2, total4 = g.H * g.W * cv;
    for (int i = tid; i < total4; i += kWinThreads) {
      const int pix = (int)fdiv((uint32_t)i, g.dCv), c4 = (i - pix * cv) * 4;
      const int hh = (int)fdiv((uint32_t)pix, g.dW), w = pix - hh * g.W;
      f4 sum = {0.f, 0.f, 0.f, 0.f};
      for (int rr = 0; rr < g.R; ++rr) {
        const int p = hh + g.pad - rr;
        if (p < 0 || p >= g.P) continue;
        for (int ss = 0; ss < g.R; ++ss) {
          const int q = w + g.pad - ss;
          if (q < 0 || q >= g.Q) continue;
          sum += *(const f4 *)&colS[(p * g.Q + q) * g.ldc + (rr * g.R + ss) * g.Cin + c4];
        }
      }
      const int o = pix * g.Cin + c4;
      if (mp) {
        const f4 m = *(const f4 *)&mp[o];
        sum.x = m.x > 0.f ? sum.x : 0.f, sum.y = m.y > 0.f ? sum.y : 0.f;
        sum.z = m.z > 0.f ? sum.z : 0.f, sum.w = m.w > 0.f ? sum.w : 0.f;
      }
      if (accumulate) sum += *(const f4 *)&op[o];
      *(f4 *)&op[o] = sum;
    }
    return;
  }
  for (int i = tid; i < total; i += kWinThreads) {
    const int pix = (int)fdiv((uint32_t)i, g.dCin), ci = i - pix * g.Cin;
    const int hh = (int)fdiv((uint32_t)pix, g.dW), w = pix - hh * g.W;
    float sum = 0.f;
    for (int rr = 0; rr < g.R; ++rr) {
      const int p = hh + g.pad - rr;
      if (p < 0 || p >= g.P) continue;
      for (int ss = 0; ss < g.R; ++ss) {
        const int q = w + g.pad - ss;
        if (q < 0 || q >= g.Q) continue;
        sum += colS[(p * g.Q + q) * g.ldc + (rr * g.R + ss) * g.Cin + ci];
      }
    }
    if (mp && !(mp[i] > 0.f)) sum = 0.f;
    op[i] = accumulate ? op[i] + sum : sum;
  }
}

bool make_win_geom(int B, int H, int W, int Cin, int Cout, int R, int pad, WinGeom &g) {
  g.B = B, g.H = H, g.W = W, g.Cin = Cin, g.Cout = Cout, g.R = R, g.pad = pad;
  g.P = H + 2 * pad - R + 1, g.Q = W + 2 * pad - R + 1;
  if (g.P < 1 || g.Q < 1 || g.P * g.Q > kWinMaxPix || Cout > kWinMaxCout || Cout < 1) return false;
  g.NC = R * R * Cin;
  g.KG = (Cout + 7) / 8;
  g.lda = win_lda(Cout);
  g.vec = Cin % 4 == 0;
  g.ldc = g.vec ? g.NC + 4 : g.NC + 1;
  g.dCin = make_fastdiv(Cin), g.dW = make_fastdiv(W), g.dCout = make_fastdiv(Cout);
  g.dCv = make_fastdiv(g.vec ? Cin / 4 : 1);
  const long long lds = ((long long)kWinMaxPix * g.lda + (long long)g.P * g.Q * g.ldc) * 4;
  return lds <= kWinLdsBytes && (long long)B * H * W * Cin < (1LL << 31);
}

}  // namespace

bool dgrad_window_applicable(int dtype, int B, int H, int W, int Cin, int Cout, int R, int stride, int pad) {
  WinGeom g;
  return dtype == 0 && stride == 1 && R > 1 && B >= 1 && B <= 65535 && make_win_geom(B, H, W, Cin, Cout, R, pad, g);
}

hipError_t launch_dgrad_window(hipStream_t st, int n, int B, int H, int W, int Cin, int Cout, int R, int pad,
                               const float *dy, long long dy_rs, const float *w, long long w_rs,
                               const float *mask, long long mask_rs, int accumulate, float *dx, long long dx_rs) {
  WinGeom g;
  if (!make_win_geom(B, H, W, Cin, Cout, R, pad, g) || n < 1 || n > 65535 || B > 65535) return hipErrorInvalidValue;
  if (!aligned_to(dy, 16)) return hipErrorInvalidValue;
  const size_t lds = ((size_t)kWinMaxPix * g.lda + (size_t)g.P * g.Q * g.ldc) * sizeof(float);
  static bool raised = false;   // more than 64 KB of dynamic LDS has to be asked for once
  if (!raised) {
    hipError_t e = hipFuncSetAttribute((const void *)k_dgrad_window, hipFuncAttributeMaxDynamicSharedMemorySize, kWinLdsBytes);
    if (e != hipSuccess) return e;
    raised = true;
  }
  hipLaunchKernelGGL(k_dgrad_window, dim3(B, n), dim3(kWinThreads), lds, st, g, dy, dy_rs, w, w_rs, mask,
                     mask_rs, accumulate, dx, dx_rs);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Backward-weight of the same kind of layer (fp32, stride 1, images of at most 64 output pixels), the window
// gather done in LDS:   dW[n][(r, s, ci)] = sum over images and output pixels m of dy[m][n] * x[m + (r, s)][ci].
// A workgroup takes a few images one after the other; per image the input patch (12 x 12 x 20 floats for LeNet's
// second convolution) and the dy tile lie in LDS, and both MFMA operands are read from there element by element:
// the (tap, channel) column of a lane is a fixed offset into the patch, the pixel a wavefront-uniform base.  In the
// generic kernel the same gather runs against global memory, 25 times per input element.  Eight wavefronts own
// the 2 x 16 tiles of 32 x 32 outputs (two column tiles and both row tiles each); the partial sums of the
// workgroups are added by the fixed-order reduction every split backward-weight kernel uses.
// ---------------------------------------------------------------------------------------------
namespace {

constexpr int kWgwMaxPatch = 6144;  // floats of one padded input patch

struct WgWinGeom {
  int B, H, W, Cin, Cout, R, pad, P, Q, NC;
  int Hp, Wp;       // padded patch
  int ipw;          // images per workgroup
  int lda;          // pitch of the dy tile
  FastDiv dQ, dCin, dR, dW, dCout;
};

__global__ __launch_bounds__(kWinThreads) void k_wgrad_window(const WgWinGeom g, const float *__restrict__ dy,
                                                              long long dy_rs, const float *__restrict__ x,
                                                              long long x_rs, float *__restrict__ out, long long out_rs,
                                                              long long split_stride) {
  __shared__ __attribute__((aligned(16))) float xS[kWgwMaxPatch];
  __shared__ __attribute__((aligned(16))) float dyS[kWinMaxPix * (kWinMaxCout + 4)];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x, rep = blockIdx.y;
  const int PQ = g.P * g.Q, patch = g.Hp * g.Wp * g.Cin, img_x = g.H * g.W * g.Cin;
  const int b_begin = split * g.ipw, b_end = min(g.B, b_begin + g.ipw);
  const float *xp = x + rep * x_rs, *dyp = dy + rep * dy_rs;
  const int r = lane & 31, h = lane >> 5;

  // this lane's two columns (tap, channel): offset into the patch from the pixel's window origin
  int off[2];
  bool ok[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int col = (2 * wave + t) * 32 + r;
    ok[t] = col < g.NC;
    const int tapi = (int)fdiv((uint32_t)(ok[t] ? col : 0), g.dCin), ci = (ok[t] ? col : 0) - tapi * g.Cin;
    const int dr = (int)fdiv((uint32_t)tapi, g.dR), ds = tapi - dr * g.R;
    off[t] = (dr * g.Wp + ds) * g.Cin + ci;
  }
  f16v acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][t][v] = 0.f;

  // zero once: the patch border (padding) and the rows / columns of the dy tile beyond the image stay zero
  for (int i = tid; i < patch; i += kWinThreads) xS[i] = 0.f;
  for (int i = tid; i < kWinMaxPix * g.lda; i += kWinThreads) dyS[i] = 0.f;

  constexpr int XI = (kWgwMaxPatch + kWinThreads - 1) / kWinThreads, DI = (kWinMaxPix * kWinMaxCout) / kWinThreads;
  float xr[XI], dr_[DI];
  auto load_img = [&](int b) {   // global -> registers (both tensors are contiguous per image)
    const float *xi = xp + (long long)b * img_x, *di = dyp + (long long)b * PQ * g.Cout;
#pragma unroll
    for (int u = 0; u < XI; ++u) {
      const int i = u * kWinThreads + tid;
      xr[u] = (b < b_end && i < img_x) ? xi[i] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < DI; ++u) {
      const int i = u * kWinThreads + tid;
      dr_[u] = (b < b_end && i < PQ * g.Cout) ? di[i] : 0.f;
    }
  };
  auto store_img = [&]() {
#pragma unroll
    for (int u = 0; u < XI; ++u) {
      const int i = u * kWinThreads + tid;
      if (i < img_x) {
        const int pix = (int)fdiv((uint32_t)i, g.dCin), ci = i - pix * g.Cin;
        const int hh = (int)fdiv((uint32_t)pix, g.dW), ww = pix - hh * g.W;
        xS[((hh + g.pad) * g.Wp + ww + g.pad) * g.Cin + ci] = xr[u];
      }
    }
#pragma unroll
    for (int u = 0; u < DI; ++u) {
      const int i = u * kWinThreads + tid;
      if (i < PQ * g.Cout) {
        const int m = (int)fdiv((uint32_t)i, g.dCout), k = i - m * g.Cout;
        dyS[m * g.lda + k] = dr_[u];
      }
    }
  };

  load_img(b_begin);
  for (int b = b_begin; b < b_end; ++b) {
    __syncthreads();  // the previous image has been multiplied (first trip: the zeros are in place)
    store_img();
    __syncthreads();
    load_img(b + 1);
    for (int q = 0; q < (PQ + 7) / 8; ++q) {
      // fragment element j of half h: pixel m = 8q + 4h + j (pixels beyond the image meet zero rows of dy)
      u4 af[2], bf[2];
      float av[2][4], bv[2][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int m = 8 * q + 4 * h + j, mc = m < PQ ? m : PQ - 1;
        const int p = (int)fdiv((uint32_t)mc, g.dQ), qq = mc - p * g.Q;
        const int base = (p * g.Wp + qq) * g.Cin;
#pragma unroll
        for (int a = 0; a < 2; ++a) av[a][j] = dyS[m * g.lda + a * 32 + r];
#pragma unroll
        for (int t = 0; t < 2; ++t) bv[t][j] = ok[t] ? xS[base + off[t]] : 0.f;
      }
#pragma unroll
      for (int a = 0; a < 2; ++a)
        af[a] = u4{__float_as_uint(av[a][0]), __float_as_uint(av[a][1]), __float_as_uint(av[a][2]), __float_as_uint(av[a][3])};
#pragma unroll
      for (int t = 0; t < 2; ++t)
        bf[t] = u4{__float_as_uint(bv[t][0]), __float_as_uint(bv[t][1]), __float_as_uint(bv[t][2]), __float_as_uint(bv[t][3])};
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int t = 0; t < 2; ++t) mma<float>(af[a], bf[t], acc[a][t]);
    }
  }
  // accumulator v of a lane: row (output channel) 8*(v/4) + 4*h + v%4 of its row tile, column r of its column tile
  float *op = out + rep * out_rs + split * split_stride;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int col = (2 * wave + t) * 32 + r;
      if (col >= g.NC) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int n = a * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (n < g.Cout) op[(long long)n * g.NC + col] = acc[a][t][v];
      }
    }
}

bool make_wgwin_geom(const ConvGeom &cg, WgWinGeom &g) {
  if (cg.sp != 1 || cg.sr != 1 || cg.dshift != 0 || cg.R != cg.S || cg.R < 2) return false;
  const int PQ = cg.P * cg.Q;
  if (PQ > kWinMaxPix || PQ % 8 != 0 || cg.N > kWinMaxCout || cg.M % PQ != 0) return false;
  g.B = cg.M / PQ, g.H = cg.Hin, g.W = cg.Win, g.Cin = cg.Cc, g.Cout = cg.N, g.R = cg.R, g.pad = -cg.off;
  g.P = cg.P, g.Q = cg.Q, g.NC = cg.K;
  if (g.pad < 0 || g.NC > 512 || g.NC < 128) return false;
  g.Hp = g.H + 2 * g.pad, g.Wp = g.W + 2 * g.pad;
  if ((long long)g.Hp * g.Wp * g.Cin > kWgwMaxPatch) return false;
  g.lda = kWinMaxCout + 4;
  g.dQ = make_fastdiv(g.Q), g.dCin = make_fastdiv(g.Cin), g.dR = make_fastdiv(g.R), g.dW = make_fastdiv(g.W);
  g.dCout = make_fastdiv(g.Cout);
  return true;
}

// images per workgroup: about one workgroup per compute unit, rows per split a multiple of 32
int wgwin_images_per_wg(const WgWinGeom &g, int replicas) {
  int ipw = (int)(((long long)g.B * replicas + 255) / 256);
  if (ipw < 1) ipw = 1;
  while ((ipw * g.P * g.Q) % 32 != 0) ++ipw;
  return ipw;
}

}  // namespace

bool wgrad_window_applicable(int dtype, const ConvGeom &g) {
  WgWinGeom wg;
  return dtype == 0 && make_wgwin_geom(g, wg);
}

int wgrad_window_plan(int replicas, const ConvGeom &g, int *chunk_out) {
  WgWinGeom wg;
  make_wgwin_geom(g, wg);
  const int ipw = wgwin_images_per_wg(wg, replicas);
  if (chunk_out) *chunk_out = ipw * wg.P * wg.Q;
  return (wg.B + ipw - 1) / ipw;
}

hipError_t launch_wgrad_window(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io) {
  WgWinGeom wg;
  if (!make_wgwin_geom(g, wg)) return hipErrorInvalidValue;
  const int PQ = wg.P * wg.Q;
  if (io.chunk % PQ != 0 || io.chunk < PQ) return hipErrorInvalidValue;
  wg.ipw = io.chunk / PQ;
  if ((long long)wg.ipw * io.splits < wg.B) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_wgrad_window, dim3(io.splits, replicas), dim3(kWinThreads), 0, st, wg, (const float *)io.dy, io.dy_rs,
                     (const float *)io.x, io.x_rs, io.out, io.out_rs, io.split_stride);
  return hipGetLastError();
}
