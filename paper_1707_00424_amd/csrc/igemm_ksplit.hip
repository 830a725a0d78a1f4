// Plain matrix products with few output tiles and a long contraction (the fully connected layers of the MLP,
// of LeNet and at the end of the residual networks; forward and backward-data): out[m][n] = sum_k in[m][k] w[n][k].
//
// With a handful of 64 x 64 tiles the staged kernels run one workgroup per compute unit on a fraction of the
// chip, and every contraction step then costs its full round trip (load, LDS, barrier, MFMA, barrier), about
// half a microsecond, tens of steps in a row.  Here a workgroup owns one 32 x 32 output tile and its four
// wavefronts split the contraction between them.  A wavefront's MFMA fragments are 16-byte pieces of a row of
// `in` and of a row of `w`, which is what one buffer load per lane fetches, so it runs from registers with no
// LDS tile and no barrier, several steps of loads in flight; the four partial tiles meet in LDS once, are
// added in wavefront order, and wavefront 0 writes the result through the common epilogue.
#include "igemm_dev.h"

namespace {

using namespace igemm_dev;

constexpr uint32_t kOob = 0x80000000u;

template <typename T, bool OUT_F32>
__global__ __launch_bounds__(kThreads) void k_gemm_ksplit(const ConvGeom g, const GemmIO io) {
  constexpr int VW = 16 / sizeof(T);  // elements per fragment: lane half h holds k = 2*VW*s + VW*h .. +VW-1 of sub-step s
  constexpr int KS = 2 * VW;          // contraction elements per sub-step
  constexpr int U = 4;                // sub-steps in flight
  __shared__ __attribute__((aligned(16))) float part[3][64 * 16];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = blockIdx.z, m0 = blockIdx.x * 32, n0 = blockIdx.y * 32;
  const int row_l = lane & 31, h = lane >> 5;
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.in + rep * io.in_rs), 0, (int)(io.in_bytes), 0x00020000);
  const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.w + rep * io.w_rs), 0, (int)((long long)g.N * g.K * sizeof(T)), 0x00020000);

  // this wavefront's quarter of the contraction, in whole sub-steps
  const int subs = (g.K + KS - 1) / KS, per = (subs + 3) / 4;
  const int s_begin = wave * per, s_end = min(subs, s_begin + per);
  const int m = m0 + row_l, n = n0 + row_l;
  const uint32_t a_row = m < g.M ? (uint32_t)((m * g.K + VW * h) * (int)sizeof(T)) : kOob;
  const uint32_t b_row = n < g.N ? (uint32_t)((n * g.K + VW * h) * (int)sizeof(T)) : kOob;

  f16v acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  for (int s0 = s_begin; s0 < s_end; s0 += U) {
    u4 af[U], bf[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // K is a multiple of VW, so a fragment lies inside the row or beyond it (and beyond this quarter)
      const int k = (s0 + u) * KS + VW * h;
      const bool ok = s0 + u < s_end && k < g.K;
      const uint32_t kb = (uint32_t)((s0 + u) * KS * (int)sizeof(T));
      af[u] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, ok && a_row != kOob ? a_row + kb : kOob, 0, 0);
      bf[u] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, ok && b_row != kOob ? b_row + kb : kOob, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) mma<T>(af[u], bf[u], acc);
  }

  // partial tiles of wavefronts 1..3 to LDS; wavefront 0 adds them in order and finishes the tile
  if (wave) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *(f4 *)&part[wave - 1][lane * 16 + q * 4] = f4{acc[q * 4], acc[q * 4 + 1], acc[q * 4 + 2], acc[q * 4 + 3]};
  }
  __syncthreads();
  if (wave) return;
#pragma unroll
  for (int w = 0; w < 3; ++w)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f4 p = *(const f4 *)&part[w][lane * 16 + q * 4];
      acc[q * 4] += p.x, acc[q * 4 + 1] += p.y, acc[q * 4 + 2] += p.z, acc[q * 4 + 3] += p.w;
    }
  f16v tile[1][1] = {{acc}};
  store_tile<T, 1, 1, OUT_F32>(g, io, rep, m0, n0, lane, tile);
}

template <typename T>
hipError_t run_ksplit(hipStream_t st, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io) {
  dim3 grid((g.M + 31) / 32, (g.N + 31) / 32, replicas);
  if (out_f32)
    hipLaunchKernelGGL((k_gemm_ksplit<T, true>), grid, dim3(kThreads), 0, st, g, io);
  else
    hipLaunchKernelGGL((k_gemm_ksplit<T, false>), grid, dim3(kThreads), 0, st, g, io);
  return hipGetLastError();
}

}  // namespace

// A plain product (1 x 1 window, stride 1, no padding: row m of the product reads row m of `in`) whose 64 x 64
// tiles would leave the chip at one workgroup per compute unit or less, with a contraction long enough to split.
bool gemm_ksplit_applicable(int dtype, int replicas, const ConvGeom &g, const GemmIO &io) {
  const int vw = dtype ? 8 : 4;
  if (g.R != 1 || g.S != 1 || g.sp != 1 || g.off != 0 || g.dshift != 0 || g.Hin != g.P || g.Win != g.Q) return false;
  if (!io.vecA || !io.vecB || g.K % vw != 0 || g.K < 8 * vw) return false;
  if (io.in_bytes <= 0 || io.in_bytes >= (1LL << 31) || (long long)g.N * g.K * (dtype ? 2 : 4) >= (1LL << 31)) return false;
  const long long tiles64 = (long long)((g.M + 63) / 64) * ((g.N + 63) / 64) * replicas;
  return tiles64 <= 256;
}

hipError_t launch_gemm_ksplit(hipStream_t st, int dtype, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io) {
  return dtype ? run_ksplit<bf16_t>(st, out_f32, replicas, g, io) : run_ksplit<float>(st, out_f32, replicas, g, io);
}

// ---------------------------------------------------------------------------------------------
// fp32 backward-weight of a first layer: at most 32 output channels and a whole window of at most 32 values
// (LeNet's first convolution: 20 x 25).  The result is one 32 x 32 MFMA tile; the generic kernel would multiply
// a 64 x 64 tile of mostly padding.  A workgroup takes the rows of one split, its four wavefronts a quarter
// each; an MFMA (32 x 32 x 2) contracts two rows, whose operands are one float of dy and one gathered float of
// the input per lane, loaded straight into registers (the window position of a lane is fixed, its pixel
// advances by two per MFMA).  The four partial tiles are added in wavefront order.
// With io.with_bias (window of fewer than 32 values) the first unused column of the x operand is all ones: that
// column of the result is sum_m dy[m][n], the bias gradient, at no cost; it goes behind the N*K values.
// ---------------------------------------------------------------------------------------------
namespace {

__global__ __launch_bounds__(kThreads) void k_wgrad_small_f32(const ConvGeom g, const WgradIO io) {
  __shared__ __attribute__((aligned(16))) float part[3][64 * 16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = blockIdx.z / io.splits, split = blockIdx.z % io.splits;
  const int col = lane & 31, h = lane >> 5;  // output channel n (operand dy) and window value k (operand x)
  const float *dy = (const float *)io.dy + rep * io.dy_rs;
  const float *x = (const float *)io.x + rep * io.x_rs;
  // rows of this wavefront: a quarter of the split, in pairs
  const int r_begin = split * io.chunk, r_end = min(g.M, r_begin + io.chunk);
  const int quarter = ((r_end - r_begin + 7) / 8) * 2;  // even
  const int m0 = r_begin + wave * quarter, m1 = min(r_end, m0 + quarter);
  // window position of this lane
  const bool k_ok = col < g.K, n_ok = col < g.N;
  const int kk = k_ok ? col : 0;
  const int rs = (int)fdiv((uint32_t)kk, g.dCc), kc = kk - rs * g.Cc;
  const int kr = (int)fdiv((uint32_t)rs, g.dS), ks = rs - kr * g.S;
  // pixel of row m0 + h
  const int PQ = g.P * g.Q;
  int m = m0 + h;
  const uint32_t mm = m < g.M ? m : 0;
  int b = (int)fdiv(mm, g.dPQ), rem = (int)mm - b * PQ;
  int p = (int)fdiv((uint32_t)rem, g.dQ), q = rem - p * g.Q;

  f16v acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  // operands of U MFMAs per batch; the next batch is requested before the current one is multiplied
  constexpr int U = 8;
  auto load_batch = [&](float (&av)[U], float (&bv)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool live = m < m1;
      const int ih = p * g.sp + g.off + kr, iw = q * g.sp + g.off + ks;
      const bool tap_ok = ih >= 0 && ih < g.Hin && iw >= 0 && iw < g.Win;
      av[u] = (live && n_ok) ? dy[(long long)m * g.N + col] : 0.f;
      bv[u] = (live && k_ok && tap_ok) ? x[((long long)(b * g.Hin + ih) * g.Win + iw) * g.Cc + kc] : 0.f;
      if (io.with_bias && col == g.K) bv[u] = live ? 1.f : 0.f;
      m += 2, q += 2;
      while (q >= g.Q) {
        q -= g.Q;
        if (++p == g.P) p = 0, ++b;
      }
    }
  };
  float a0[U], b0[U], a1[U], b1[U];
  load_batch(a0, b0);
  for (int mj = m0; mj < m1; mj += 4 * U) {
    load_batch(a1, b1);  // rows at or beyond m1 load nothing
#pragma unroll
    for (int u = 0; u < U; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[u], b0[u], acc, 0, 0, 0);
    load_batch(a0, b0);
#pragma unroll
    for (int u = 0; u < U; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[u], b1[u], acc, 0, 0, 0);
  }
  if (wave) {
#pragma unroll
    for (int qd = 0; qd < 4; ++qd)
      *(f4 *)&part[wave - 1][lane * 16 + qd * 4] = f4{acc[qd * 4], acc[qd * 4 + 1], acc[qd * 4 + 2], acc[qd * 4 + 3]};
  }
  __syncthreads();
  if (wave) return;
#pragma unroll
  for (int w = 0; w < 3; ++w)
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      const f4 t = *(const f4 *)&part[w][lane * 16 + qd * 4];
      acc[qd * 4] += t.x, acc[qd * 4 + 1] += t.y, acc[qd * 4 + 2] += t.z, acc[qd * 4 + 3] += t.w;
    }
  // register v of a lane: output channel n = 8*(v/4) + 4*h + v%4, window value k = col
  float *out = io.out + rep * io.out_rs + split * io.split_stride;
  if (k_ok) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int n = 8 * (v >> 2) + 4 * h + (v & 3);
      if (n < g.N) out[(long long)n * g.K + col] = acc[v];
    }
  } else if (io.with_bias && col == g.K) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int n = 8 * (v >> 2) + 4 * h + (v & 3);
      if (n < g.N) out[(long long)g.N * g.K + n] = acc[v];
    }
  }
}

}  // namespace

bool wgrad_small_f32_applicable(int dtype, const ConvGeom &g) {
  return dtype == 0 && g.K <= 32 && g.N <= 32 && g.dshift == 0 && g.sr == 1 && g.M >= 1 && g.Q >= 1;
}

hipError_t launch_wgrad_small_f32(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io) {
  dim3 grid(1, 1, replicas * io.splits);
  hipLaunchKernelGGL(k_wgrad_small_f32, grid, dim3(kThreads), 0, st, g, io);
  return hipGetLastError();
}
