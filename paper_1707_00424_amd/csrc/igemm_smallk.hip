// Forward convolution of a layer whose whole contraction fits one LDS tile: K = R*S*Cin <= 32
// (the first layer of each network: 1 or 3 input channels).
//
// Such a layer is bound by the gather of its operand and by its output stream, not by the matrix
// units, and the generic kernel spends most of its time in per-workgroup fixed costs on 64- or
// 128-row tiles.  Here a workgroup owns 256 output pixels: every thread gathers the K values of
// ONE pixel (tap offsets are wavefront-uniform, so the address of a value is the pixel's base plus
// a scalar), packs them into a row of the operand tile in LDS, the weights [N][K] are padded to
// [N][32] in LDS, one barrier, a handful of MFMAs per wavefront, and the row-contiguous epilogue
// shared with the other kernels.
#include "igemm_dev.h"

namespace {

using namespace igemm_dev;

constexpr int kKP = 32;  // padded contraction length

// one element through a raw buffer load: an offset beyond the buffer returns zero
template <typename T>
__device__ __forceinline__ T buffer_load_elem(__amdgpu_buffer_rsrc_t rsrc, uint32_t off);
template <>
__device__ __forceinline__ bf16_t buffer_load_elem<bf16_t>(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
  return (bf16_t)__builtin_amdgcn_raw_buffer_load_b16(rsrc, off, 0, 0);
}
template <>
__device__ __forceinline__ float buffer_load_elem<float>(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
  return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, off, 0, 0));
}

// STAT: also the column sums of the output for the batch-norm behind the layer (see store_tile_lds), one partial
// row per workgroup.  (The 64-wide bf16 variant came out at 172 registers, four over the budget of three wavefronts
// per SIMD: it is held to that budget.)
// IN_F32 (bf16 layers): the gathered tensor is fp32 in memory, rounded to bf16 as it is gathered.
template <typename T, int TN, bool OUT_F32, bool STAT, bool IN_F32 = false>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(sizeof(T) == 2 && TN == 2 && !OUT_F32 ? 3 : 1))) void k_conv_smallk(const ConvGeom g, const GemmIO io) {
  static_assert(!IN_F32 || sizeof(T) == 2, "fp32 layers read fp32 as it is");
  constexpr int VW = 16 / sizeof(T);
  constexpr int BK = 4 * VW;               // one contraction step of the MFMA helper: 32 bf16 / 16 fp32
  constexpr int STEPS = kKP / BK;          // 1 / 2
  constexpr int LK = BK + VW;
  constexpr int TM = 2, BM = 256, BN = TN * 32;
  constexpr int kTileBytes = STEPS * (BM + BN) * LK * (int)sizeof(T);
  constexpr int kStageBytes = (4 * kStageFloats<TN> + (STAT ? 4 * 2 * BN : 0)) * (int)sizeof(float);
  __shared__ __attribute__((aligned(16))) char smem[kTileBytes > kStageBytes ? kTileBytes : kStageBytes];
  T *As = reinterpret_cast<T *>(smem);                                   // [STEPS][BM][LK]
  T *Bs = reinterpret_cast<T *>(smem) + STEPS * BM * LK;                 // [STEPS][BN][LK]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = blockIdx.z;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  constexpr int IS = IN_F32 ? 4 : (int)sizeof(T);  // bytes per gathered element in memory
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const char *)io.in + rep * io.in_rs * IS), 0, (int)(io.in_bytes), 0x00020000);
  const T *__restrict__ w = (const T *)io.w + rep * io.w_rs;

  // this thread's pixel
  const int m = m0 + tid;
  const bool m_ok = m < g.M;
  const uint32_t mm = m_ok ? m : 0;
  const int b = fdiv(mm, g.dPQ), rem = mm - b * g.P * g.Q;
  const int p = fdiv(rem, g.dQ), q = rem - p * g.Q;
  const int h0 = p * g.sp + g.off, w0 = q * g.sp + g.off;
  const int base = ((b * g.Hin + h0) * g.Win + w0) * g.Cc;  // element offset of tap (0, 0), channel 0 (may be negative)

  // gather: value k = (r, s, c) sits at base + (r*Win + s)*Cc + c when the tap is inside the image
  T vals[kKP];
  {
    int r = 0, s = 0, c = 0;  // wavefront-uniform
#pragma unroll
    for (int k = 0; k < kKP; ++k) {
      const bool live = k < g.K;
      const bool ok = live && m_ok && (unsigned)(h0 + r) < (unsigned)g.Hin && (unsigned)(w0 + s) < (unsigned)g.Win;
      const uint32_t off = ok ? (uint32_t)((base + (r * g.Win + s) * g.Cc + c) * IS) : kOobOffset;
      if constexpr (IN_F32)
        vals[k] = (T)f32_to_bf16(buffer_load_elem<float>(a_rsrc, off));
      else
        vals[k] = buffer_load_elem<T>(a_rsrc, off);
      if (++c == g.Cc) {
        c = 0;
        if (++s == g.S) s = 0, ++r;
      }
    }
  }
  // weights: element (n, k) of [N][K] -> Bs[k / BK][n][k % BK], zero beyond N or K
  constexpr int W_IT = BN * kKP / kThreads;
  T wv[W_IT];
#pragma unroll
  for (int i = 0; i < W_IT; ++i) {
    const int e = i * kThreads + tid, n = e / kKP, k = e - n * kKP;
    wv[i] = (n0 + n < g.N && k < g.K) ? w[(long long)(n0 + n) * g.K + k] : (T)0;
  }
#pragma unroll
  for (int st = 0; st < STEPS; ++st)
#pragma unroll
    for (int v = 0; v < BK / VW; ++v) *(u4 *)&As[(st * BM + tid) * LK + v * VW] = pack_vec<T, VW>(&vals[st * BK + v * VW]);
#pragma unroll
  for (int i = 0; i < W_IT; ++i) {
    const int e = i * kThreads + tid, n = e / kKP, k = e - n * kKP;
    Bs[((k / BK) * BN + n) * LK + k % BK] = wv[i];
  }
  __syncthreads();

  f16v acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;
#pragma unroll
  for (int st = 0; st < STEPS; ++st)
    mma_tile_t<T, TM, TN, LK, VW>(As + st * BM * LK, Bs + st * BN * LK, wave * TM * 32, 0, lane, acc);
  __syncthreads();  // operand tiles are dead: their LDS becomes the staging strips
  float *wsums = reinterpret_cast<float *>(smem) + 4 * kStageFloats<TN>;
  store_tile_lds<T, TM, TN, OUT_F32, STAT>(g, io, rep, m0 + wave * TM * 32, n0, lane, acc,
                                           reinterpret_cast<float *>(smem) + wave * kStageFloats<TN>,
                                           wsums + wave * 2 * BN);
  if (STAT) write_tile_sums<BN, 4>(g, io, rep, gridDim.x, blockIdx.x, n0, tid, wsums);
}

// ---------------------------------------------------------------------------------------------
// backward-weight of such a layer (bf16): out[n, k] = sum_m dy[m, n] * gather(m, k), K <= 32.
// The output is tiny (N x 32) and the kernel streams dy once: 16-byte loads of dy rows into LDS as
// they lie in memory, the gathered operand built element by element (every thread owns four
// consecutive k of one pixel per step, tap offsets fixed per thread), MFMA fragments fetched with the
// LDS transpose read.  The contraction is split over workgroups; a second kernel adds the partials.
// ---------------------------------------------------------------------------------------------
typedef short s4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u4 tr_frag16(const bf16_t *tile, int ld, int krow, int col) {
  const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v *)(tile + krow * ld + col));
  const s4v hi =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s4v *)(tile + (krow + 4) * ld + col));
  u4 r;
  r.x = (uint32_t)(unsigned short)lo.x | ((uint32_t)(unsigned short)lo.y << 16);
  r.y = (uint32_t)(unsigned short)lo.z | ((uint32_t)(unsigned short)lo.w << 16);
  r.z = (uint32_t)(unsigned short)hi.x | ((uint32_t)(unsigned short)hi.y << 16);
  r.w = (uint32_t)(unsigned short)hi.z | ((uint32_t)(unsigned short)hi.w << 16);
  return r;
}

template <bool X_F32>
__global__ __launch_bounds__(kThreads) void k_wgrad_smallk(const ConvGeom g, const WgradIO io) {
  constexpr int BKM = 32;             // pixels per contraction step
  constexpr int BM = 128, BN = kKP;   // output tile: 128 output channels (four wavefronts) x 32 contraction columns
  constexpr int LDA = BM + 16, LDB = BN + 16;
  constexpr int AV = BM / 8;          // 16-byte vectors per dy pixel row
  constexpr int A_IT = BKM * AV / kThreads;
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BKM * LDA];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BKM * LDB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = blockIdx.z / io.splits, split = blockIdx.z % io.splits;
  const int n0 = blockIdx.y * BM;
  const int m_begin = split * io.chunk, m_end = min(g.M, m_begin + io.chunk);
  const int PQ = g.P * g.Q;
  constexpr int XS = X_F32 ? 4 : 2;  // bytes per element of x in memory
  const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const char *)io.x + rep * io.x_rs * XS), 0, (int)((long long)(g.M / PQ) * g.Hin * g.Win * g.Cc * XS), 0x00020000);
  const __amdgpu_buffer_rsrc_t d_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const bf16_t *)io.dy + rep * io.dy_rs), 0, (int)((long long)g.M * g.N * 2), 0x00020000);

  // gathered operand: this thread's pixel inside a step and its four columns k = 4*(tid%8) .. +3
  const int bpx = tid >> 3, kq = (tid & 7) * 4;
  int k_off[4], k_r[4], k_s[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int k = kq + e;
    const uint32_t kk = k < g.K ? k : 0;
    const uint32_t rs = fdiv(kk, g.dCc);
    const int c = kk - rs * g.Cc;
    k_r[e] = k < g.K ? (int)fdiv(rs, g.dS) : -100000;   // never a valid row
    k_s[e] = rs - fdiv(rs, g.dS) * g.S;
    k_off[e] = ((int)fdiv(rs, g.dS) * g.Win + k_s[e]) * g.Cc + c;
  }
  // dy: vector v = it*256 + tid -> pixel v / AV, channels 8*(v % AV) .. +7
  auto load_tiles = [&](int mbase, u4 (&areg)[A_IT], unsigned short (&breg)[4]) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int v = i * kThreads + tid, row = v / AV, cv = v % AV;
      const int m = mbase + row, n = n0 + cv * 8;
      const bool ok = m < m_end && n < g.N;
      areg[i] = __builtin_amdgcn_raw_buffer_load_b128(d_rsrc, ok ? (uint32_t)((m * g.N + n) * 2) : kOobOffset, 0, 0);
    }
    const int m = mbase + bpx;
    const bool mok = m < m_end;
    const uint32_t mm = mok ? m : 0;
    const int b = fdiv(mm, g.dPQ), rem = mm - b * PQ;
    const int p = fdiv(rem, g.dQ), q = rem - p * g.Q;
    const int h0 = p * g.sp + g.off, w0 = q * g.sp + g.off;
    const int base = ((b * g.Hin + h0) * g.Win + w0) * g.Cc;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool ok = mok && (unsigned)(h0 + k_r[e]) < (unsigned)g.Hin && (unsigned)(w0 + k_s[e]) < (unsigned)g.Win;
      const uint32_t xo = ok ? (uint32_t)((base + k_off[e]) * XS) : kOobOffset;
      if constexpr (X_F32)
        breg[e] = f32_to_bf16(__uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(x_rsrc, xo, 0, 0)));
      else
        breg[e] = __builtin_amdgcn_raw_buffer_load_b16(x_rsrc, xo, 0, 0);
      // the first unused column is all ones over the live pixels: its products are the column sums of dy
      if (io.with_bias && kq + e == g.K) breg[e] = mok ? (unsigned short)0x3F80 : (unsigned short)0;
    }
  };
  auto store_tiles = [&](int buf, const u4 (&areg)[A_IT], const unsigned short (&breg)[4]) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int v = i * kThreads + tid;
      *(u4 *)&As[buf][(v / AV) * LDA + (v % AV) * 8] = areg[i];
    }
    typedef unsigned int u2v __attribute__((ext_vector_type(2)));
    const u2v pk = {(uint32_t)breg[0] | ((uint32_t)breg[1] << 16), (uint32_t)breg[2] | ((uint32_t)breg[3] << 16)};
    *(u2v *)&Bs[buf][bpx * LDB + kq] = pk;
  };

  f16v acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const int gq = lane >> 4, j = lane & 15;
  const int frag_k = 8 * (gq >> 1) + (j >> 2), frag_c = 16 * (gq & 1) + 4 * (j & 3);
  auto mma_step = [&](const bf16_t *at, const bf16_t *bt) {
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const u4 af = tr_frag16(at, LDA, sub * 16 + frag_k, wave * 32 + frag_c);
      const u4 bf = tr_frag16(bt, LDB, sub * 16 + frag_k, frag_c);
      mma<bf16_t>(af, bf, acc);
    }
  };
  // two-step-deep software pipeline (rows at or beyond m_end load zeros); an empty split writes zeros
  const int KT = m_end > m_begin ? (m_end - m_begin + BKM - 1) / BKM : 0;
  u4 a0[A_IT], a1[A_IT];
  unsigned short b0[4], b1[4];
  load_tiles(m_begin, a0, b0);
  load_tiles(m_begin + BKM, a1, b1);
  store_tiles(0, a0, b0);
  __syncthreads();
  int kt = 0;
  for (; kt + 1 < KT; kt += 2) {
    load_tiles(m_begin + (kt + 2) * BKM, a0, b0);
    mma_step(As[0], Bs[0]);
    store_tiles(1, a1, b1);
    __syncthreads();
    load_tiles(m_begin + (kt + 3) * BKM, a1, b1);
    mma_step(As[1], Bs[1]);
    store_tiles(0, a0, b0);
    __syncthreads();
  }
  if (kt < KT) mma_step(As[0], Bs[0]);

  float *out = io.out + rep * io.out_rs + split * io.split_stride;
  const int k = lane & 31, h = lane >> 5;
  if (k < g.K) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int n = n0 + wave * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
      if (n < g.N) out[(long long)n * g.K + k] = acc[v];
    }
  } else if (io.with_bias && k == g.K) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int n = n0 + wave * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
      if (n < g.N) out[(long long)g.N * g.K + n] = acc[v];
    }
  }
}

template <typename T, int TN>
hipError_t run_smallk(hipStream_t st, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io) {
  dim3 grid((g.M + 255) / 256, (g.N + TN * 32 - 1) / (TN * 32), replicas);
  if (io.in_f32) {  // a bf16 layer over fp32 memory
    if constexpr (sizeof(T) == 2) {
      if (out_f32 || (io.stat && TN > 2)) return hipErrorInvalidValue;
      if (io.stat)
        hipLaunchKernelGGL((k_conv_smallk<T, TN, false, TN <= 2, true>), grid, dim3(kThreads), 0, st, g, io);
      else
        hipLaunchKernelGGL((k_conv_smallk<T, TN, false, false, true>), grid, dim3(kThreads), 0, st, g, io);
      return hipGetLastError();
    } else {
      return hipErrorInvalidValue;
    }
  }
  if (io.stat) {
    if (TN > 2 || out_f32) return hipErrorInvalidValue;  // see conv_smallk_stat_splits
    hipLaunchKernelGGL((k_conv_smallk<T, TN, false, TN <= 2>), grid, dim3(kThreads), 0, st, g, io);
  } else if (out_f32) {
    hipLaunchKernelGGL((k_conv_smallk<T, TN, true, false>), grid, dim3(kThreads), 0, st, g, io);
  } else {
    hipLaunchKernelGGL((k_conv_smallk<T, TN, false, false>), grid, dim3(kThreads), 0, st, g, io);
  }
  return hipGetLastError();
}

}  // namespace

bool conv_smallk_applicable(int dtype, const ConvGeom &g, const GemmIO &io) {
  // (fp32 with few rows: the 8-byte gather kernel measured faster)
  // (a 1 x 1 window has one tap at offset 0: the direction of the window walk does not matter, so the
  // backward-data of a 1 x 1 stride-1 layer with few output channels qualifies as well)
  return g.K <= kKP && g.dshift == 0 && (g.sr == 1 || (g.R == 1 && g.S == 1)) && g.plq == 0 && g.N % 4 == 0 && io.ldc % 4 == 0 && g.M >= (dtype ? 64 : 256) &&
         io.in_bytes > 0 && io.in_bytes < (1LL << 31) && (long long)g.M * io.ldc * 4 < (1LL << 31);
}

// partial rows of column sums a launch with io.stat set writes (one per 256 output pixels); 0: none (the
// 96-wide epilogue does not take them)
int conv_smallk_stat_splits(const ConvGeom &g, bool out_f32) { return g.N <= 64 && !out_f32 ? (g.M + 255) / 256 : 0; }

hipError_t launch_conv_smallk(hipStream_t st, int dtype, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io) {
  const int n = g.N;
  if (dtype == 0) {
    if (n <= 32) return run_smallk<float, 1>(st, out_f32, replicas, g, io);
    if (n <= 64) return run_smallk<float, 2>(st, out_f32, replicas, g, io);
    return run_smallk<float, 3>(st, out_f32, replicas, g, io);
  }
  if (n <= 32) return run_smallk<bf16_t, 1>(st, out_f32, replicas, g, io);
  if (n <= 64) return run_smallk<bf16_t, 2>(st, out_f32, replicas, g, io);
  return run_smallk<bf16_t, 3>(st, out_f32, replicas, g, io);
}

bool wgrad_smallk_applicable(int dtype, const ConvGeom &g) {
  return dtype == 1 && g.K <= kKP && g.N % 8 == 0 && g.dshift == 0 && g.sr == 1 && (long long)g.M * g.N * 2 < (1LL << 31) &&
         (long long)(g.M / (g.P * g.Q)) * g.Hin * g.Win * g.Cc * 2 < (1LL << 31) && g.M % (g.P * g.Q) == 0;
}

hipError_t launch_wgrad_smallk(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io) {
  dim3 grid(1, (g.N + 127) / 128, replicas * io.splits);
  if (io.x_f32)
    hipLaunchKernelGGL(k_wgrad_smallk<true>, grid, dim3(kThreads), 0, st, g, io);
  else
    hipLaunchKernelGGL(k_wgrad_smallk<false>, grid, dim3(kThreads), 0, st, g, io);
  return hipGetLastError();
}
