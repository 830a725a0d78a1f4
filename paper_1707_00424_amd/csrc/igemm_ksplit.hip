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
