// Implicit-GEMM convolution kernels on MFMA for gfx950 (see igemm.h for the index conventions).
//
// Tiling: a workgroup of 4 wavefronts owns a BM x BN output tile; each wavefront owns TM x TN
// MFMA tiles of 32x32 (accumulators in registers, fp32).  The contraction runs in steps of
// BK = 64 bytes of the operand type (16 fp32 / 32 bf16); both operand tiles are staged in LDS as
// [row][BK + 16 bytes of padding] so that the 16-byte fragment reads of 8 consecutive rows hit 32
// distinct banks, and LDS is double-buffered: global loads of step t+1 are in flight while the
// MFMAs of step t run, one barrier per step.
//
// MFMA register layouts relied upon (lane l of 64):
//   A, B operands: row (resp. column) l % 32, contraction slice l / 32 (the order of the contraction
//                  elements inside a step is irrelevant as long as A and B agree, which they do
//                  because both are read from LDS with the same offsets);
//   D (32x32 fp32, 16 registers v): column l % 32, row 8*(v/4) + 4*(l/32) + v%4.
#include <stdlib.h>

#include "igemm_dev.h"

namespace {

using namespace igemm_dev;

// ---------------------------------------------------------------------------------------------
// forward / backward-data: out[m, n] = epilogue( sum_k gather(m, k) * w[n, k] )
// ---------------------------------------------------------------------------------------------
template <typename T, int WAVES_M, int WAVES_N, int TM, int TN, bool OUT_F32>
__global__ __launch_bounds__(kThreads) void k_igemm(const ConvGeom g, const GemmIO io) {
  constexpr int VW = 16 / sizeof(T);
  constexpr int BK = 4 * VW;
  constexpr int LK = BK + VW;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  constexpr int A_IT = (BM + 63) / 64, B_IT = (BN + 63) / 64;
  __shared__ __attribute__((aligned(16))) T As[2][BM * LK];
  __shared__ __attribute__((aligned(16))) T Bs[2][BN * LK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int rep = blockIdx.z;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const T *__restrict__ in = (const T *)io.in + rep * io.in_rs;
  const T *__restrict__ w = (const T *)io.w + rep * io.w_rs;
  const int lrow = tid >> 2, lkv = tid & 3;
  const int PQ = g.P * g.Q;

  int a_boff[A_IT], a_h0[A_IT], a_w0[A_IT];
  bool a_ok[A_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int row = i * 64 + lrow, m = m0 + row;
    a_ok[i] = row < BM && m < g.M;
    const uint32_t mm = a_ok[i] ? m : 0;
    const uint32_t b = fdiv(mm, g.dPQ), rem = mm - b * PQ;
    const uint32_t p = fdiv(rem, g.dQ), q = rem - p * g.Q;
    a_boff[i] = b * g.Hin * g.Win * g.Cc;
    a_h0[i] = p * g.sp + g.off;
    a_w0[i] = q * g.sp + g.off;
  }
  int kk = lkv * VW, kr, ks, kc;
  {
    const uint32_t rs = fdiv(kk, g.dCc);
    kc = kk - rs * g.Cc;
    kr = fdiv(rs, g.dS);
    ks = rs - kr * g.S;
  }

  u4 areg[A_IT], breg[B_IT];
  const u4 zero4 = {0u, 0u, 0u, 0u};

  auto load_tiles = [&]() {
    if (io.vecA) {
      const bool kok = kk < g.K;
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        int ih, iw;
        const bool ok = tap(a_h0[i] + kr * g.sr, g.dshift, g.Hin, ih) & tap(a_w0[i] + ks * g.sr, g.dshift, g.Win, iw) &
                        a_ok[i] & kok;
        areg[i] = ok ? *(const u4 *)(in + a_boff[i] + (ih * g.Win + iw) * g.Cc + kc) : zero4;
      }
    } else {
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        T tmp[VW];
#pragma unroll
        for (int e = 0; e < VW; ++e) {
          const int ke = kk + e;
          const uint32_t rs = fdiv(ke < g.K ? ke : 0, g.dCc);
          const int c = (ke < g.K ? ke : 0) - rs * g.Cc;
          const int r = fdiv(rs, g.dS), s = rs - r * g.S;
          int ih, iw;
          const bool ok = tap(a_h0[i] + r * g.sr, g.dshift, g.Hin, ih) & tap(a_w0[i] + s * g.sr, g.dshift, g.Win, iw) &
                          a_ok[i] & (ke < g.K);
          tmp[e] = ok ? in[a_boff[i] + (ih * g.Win + iw) * g.Cc + c] : (T)0;
        }
        areg[i] = pack_vec<T, VW>(tmp);
      }
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int row = i * 64 + lrow, nrow = n0 + row;
      const bool rok = row < BN && nrow < g.N;
      if (io.vecB) {
        breg[i] = (rok && kk < g.K) ? *(const u4 *)(w + (long long)nrow * g.K + kk) : zero4;
      } else {
        T tmp[VW];
#pragma unroll
        for (int e = 0; e < VW; ++e) tmp[e] = (rok && kk + e < g.K) ? w[(long long)nrow * g.K + kk + e] : (T)0;
        breg[i] = pack_vec<T, VW>(tmp);
      }
    }
  };
  auto advance_k = [&]() {
    kk += BK;
    kc += BK;
    while (kc >= g.Cc) {
      kc -= g.Cc;
      if (++ks == g.S) {
        ks = 0;
        ++kr;
      }
    }
  };
  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int row = i * 64 + lrow;
      if (BM % 64 == 0 || row < BM) *(u4 *)&As[buf][row * LK + lkv * VW] = areg[i];
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int row = i * 64 + lrow;
      if (BN % 64 == 0 || row < BN) *(u4 *)&Bs[buf][row * LK + lkv * VW] = breg[i];
    }
  };

  f16v acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

  const int KT = (g.K + BK - 1) / BK;
  load_tiles();
  store_tiles(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) {
      advance_k();
      load_tiles();
    }
    mma_tile<T, TM, TN, LK, VW>(As[buf], Bs[buf], wm * TM * 32, wn * TN * 32, lane, acc);
    if (kt + 1 < KT) store_tiles(buf ^ 1);
    __syncthreads();
  }

  store_tile<T, TM, TN, OUT_F32>(g, io, rep, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, acc);
}

// ---------------------------------------------------------------------------------------------
// backward-weight: out[n, k] = sum_{m in split} dy[m, n] * gather(m, k)   (fp32 partial per split)
// Both operands arrive contraction-major from memory; each thread loads VW consecutive rows m of a
// 4-byte column group and writes them to LDS as 16-byte contraction-contiguous fragments.
// ---------------------------------------------------------------------------------------------
// BIAS (fp32): the workgroups of the first column tile also add up the dy values they stage (a thread keeps one
// output channel) and write the bias gradient, the column sums of dy, behind the weights.
template <typename T, int WAVES_M, int WAVES_N, int TM, int TN, bool BIAS = false>
__global__ __launch_bounds__(kThreads) void k_wgrad(const ConvGeom g, const WgradIO io) {
  static_assert(!BIAS || sizeof(T) == 4, "the bias sums are taken by the fp32 form only");
  constexpr int VW = 16 / sizeof(T);
  constexpr int CP = 4 / sizeof(T);  // columns per 4-byte load
  constexpr int BK = 4 * VW;
  constexpr int LK = BK + VW;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  constexpr int A_TASKS = BM / CP * 4, B_TASKS = BN / CP * 4;
  constexpr int A_IT = (A_TASKS + kThreads - 1) / kThreads, B_IT = (B_TASKS + kThreads - 1) / kThreads;
  __shared__ __attribute__((aligned(16))) T As[2][BM * LK];
  __shared__ __attribute__((aligned(16))) T Bs[2][BN * LK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int rep = blockIdx.z / io.splits, split = blockIdx.z % io.splits;
  const int n0 = blockIdx.y * BM;  // rows of the output = output channels
  const int k0 = blockIdx.x * BN;  // columns of the output = (r, s, c)
  const T *__restrict__ dy = (const T *)io.dy + rep * io.dy_rs;
  const T *__restrict__ x = (const T *)io.x + rep * io.x_rs;
  const int m_begin = split * io.chunk;
  const int m_end = min(g.M, m_begin + io.chunk);
  const int PQ = g.P * g.Q;

  // per-thread fixed column info of the gathered operand
  int b_r[B_IT][CP], b_s[B_IT][CP], b_c[B_IT][CP];
  bool b_ok[B_IT][CP];
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    const int t = i * kThreads + tid;
    const int kp = t % (BN / CP);
#pragma unroll
    for (int e = 0; e < CP; ++e) {
      const int k = k0 + kp * CP + e;
      b_ok[i][e] = t < B_TASKS && k < g.K;
      const uint32_t kk = b_ok[i][e] ? k : 0;
      const uint32_t rs = fdiv(kk, g.dCc);
      b_c[i][e] = kk - rs * g.Cc;
      b_r[i][e] = fdiv(rs, g.dS);
      b_s[i][e] = rs - b_r[i][e] * g.S;
    }
  }

  uint32_t areg[A_IT][VW], breg[B_IT][VW];  // one 4-byte column group per contraction row
  const bool tally = BIAS && blockIdx.x == 0;
  float bsum[BIAS ? A_IT : 1];
  if (BIAS) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) bsum[i] = 0.f;
  }

  auto load_tiles = [&](int mbase) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int t = i * kThreads + tid;
      const int cp = t % (BM / CP), mg = t / (BM / CP);
      const int n = n0 + cp * CP;
#pragma unroll
      for (int j = 0; j < VW; ++j) {
        const int m = mbase + mg * VW + j;
        const bool mok = t < A_TASKS && m < m_end;
        if (sizeof(T) == 4) {
          areg[i][j] = (mok && n < g.N) ? ((const uint32_t *)dy)[(long long)m * g.N + n] : 0u;
        } else if (io.pairA) {
          areg[i][j] = (mok && n < g.N) ? *(const uint32_t *)((const unsigned short *)dy + (long long)m * g.N + n) : 0u;
        } else {
          const unsigned short *p = (const unsigned short *)dy + (long long)m * g.N + n;
          const uint32_t lo = (mok && n < g.N) ? p[0] : 0u;
          const uint32_t hi = (mok && n + 1 < g.N) ? p[1] : 0u;
          areg[i][j] = lo | (hi << 16);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int t = i * kThreads + tid;
      const int mg = t / (BN / CP);
      const int mfirst = mbase + mg * VW;
      uint32_t mm = mfirst < g.M ? mfirst : 0;
      uint32_t b = fdiv(mm, g.dPQ), rem = mm - b * PQ;
      uint32_t p = fdiv(rem, g.dQ), q = rem - p * g.Q;
#pragma unroll
      for (int j = 0; j < VW; ++j) {
        const bool mok = (mfirst + j) < m_end;
        const int boff = b * g.Hin * g.Win * g.Cc;
        const int h0 = p * g.sp + g.off, w0 = q * g.sp + g.off;
        if (sizeof(T) == 4) {
          int ih, iw;
          const bool ok = tap(h0 + b_r[i][0], 0, g.Hin, ih) & tap(w0 + b_s[i][0], 0, g.Win, iw) & mok & b_ok[i][0];
          breg[i][j] = ok ? ((const uint32_t *)x)[boff + (ih * g.Win + iw) * g.Cc + b_c[i][0]] : 0u;
        } else if (io.pairB) {
          int ih, iw;
          const bool ok = tap(h0 + b_r[i][0], 0, g.Hin, ih) & tap(w0 + b_s[i][0], 0, g.Win, iw) & mok & b_ok[i][0];
          breg[i][j] =
              ok ? *(const uint32_t *)((const unsigned short *)x + boff + (ih * g.Win + iw) * g.Cc + b_c[i][0]) : 0u;
        } else {
          uint32_t v[2] = {0u, 0u};
#pragma unroll
          for (int e = 0; e < CP; ++e) {
            int ih, iw;
            const bool ok = tap(h0 + b_r[i][e], 0, g.Hin, ih) & tap(w0 + b_s[i][e], 0, g.Win, iw) & mok & b_ok[i][e];
            v[e] = ok ? ((const unsigned short *)x)[boff + (ih * g.Win + iw) * g.Cc + b_c[i][e]] : 0u;
          }
          breg[i][j] = v[0] | (v[1] << 16);
        }
        if (++q == (uint32_t)g.Q) {
          q = 0;
          if (++p == (uint32_t)g.P) {
            p = 0;
            ++b;
          }
        }
      }
    }
  };
  auto store_one = [&](T *dst, int tasks_per_row_group, int t, const uint32_t *regs, int rows_limit) {
    const int cp = t % tasks_per_row_group, mg = t / tasks_per_row_group;
    if (sizeof(T) == 4) {
      u4 v = {regs[0], regs[1], regs[2], regs[3]};
      *(u4 *)&dst[cp * LK + mg * VW] = v;
    } else {
      u4 lo, hi;
      lo.x = (regs[0] & 0xffffu) | (regs[1] << 16);
      lo.y = (regs[2] & 0xffffu) | (regs[3] << 16);
      lo.z = (regs[4] & 0xffffu) | (regs[5] << 16);
      lo.w = (regs[6] & 0xffffu) | (regs[7] << 16);
      hi.x = (regs[0] >> 16) | (regs[1] & 0xffff0000u);
      hi.y = (regs[2] >> 16) | (regs[3] & 0xffff0000u);
      hi.z = (regs[4] >> 16) | (regs[5] & 0xffff0000u);
      hi.w = (regs[6] >> 16) | (regs[7] & 0xffff0000u);
      *(u4 *)&dst[(cp * 2) * LK + mg * VW] = lo;
      *(u4 *)&dst[(cp * 2 + 1) * LK + mg * VW] = hi;
    }
  };
  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int t = i * kThreads + tid;
      if (A_TASKS % kThreads == 0 || t < A_TASKS) store_one(As[buf], BM / CP, t, areg[i], BM);
      if (BIAS && tally) {  // masked rows and columns hold zeros
#pragma unroll
        for (int j = 0; j < VW; ++j) bsum[i] += __uint_as_float(areg[i][j]);
      }
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int t = i * kThreads + tid;
      if (B_TASKS % kThreads == 0 || t < B_TASKS) store_one(Bs[buf], BN / CP, t, breg[i], BN);
    }
  };

  f16v acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

  const int KT = m_end > m_begin ? (m_end - m_begin + BK - 1) / BK : 0;
  if (KT > 0) {
    load_tiles(m_begin);
    store_tiles(0);
  }
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) load_tiles(m_begin + (kt + 1) * BK);
    mma_tile<T, TM, TN, LK, VW>(As[buf], Bs[buf], wm * TM * 32, wn * TN * 32, lane, acc);
    if (kt + 1 < KT) store_tiles(buf ^ 1);
    __syncthreads();
  }

  float *out = io.out + rep * io.out_rs + split * io.split_stride;
  const int col_l = lane & 31, h = lane >> 5;
#pragma unroll
  for (int tn = 0; tn < TN; ++tn) {
    const int k = k0 + wn * TN * 32 + tn * 32 + col_l;
    if (k >= g.K) continue;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int n = n0 + wm * TM * 32 + tm * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (n < g.N) out[(long long)n * g.K + k] = acc[tm][tn][v];
      }
  }
  if (BIAS && tally) {
    // task t of a step holds column t % BM, rows 4 * (t / BM) .. + 3: the four row groups are added in order
    float *bs = (float *)&As[0][0];  // [4][BM]; the last step ended with a barrier
    static_assert(sizeof(As) >= 4 * BM * 4, "bias staging");
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int t = i * kThreads + tid;
      if (A_TASKS % kThreads == 0 || t < A_TASKS) bs[(t / BM) * BM + t % BM] = bsum[i];
    }
    __syncthreads();
    for (int c = tid; c < BM; c += kThreads)
      if (n0 + c < g.N) out[(long long)g.N * g.K + n0 + c] = bs[c] + bs[BM + c] + bs[2 * BM + c] + bs[3 * BM + c];
  }
}

template <typename T, int WM, int WN, int TM, int TN>
hipError_t run_igemm(hipStream_t st, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  dim3 grid((g.M + BM - 1) / BM, (g.N + BN - 1) / BN, replicas);
  if (out_f32)
    hipLaunchKernelGGL((k_igemm<T, WM, WN, TM, TN, true>), grid, dim3(kThreads), 0, st, g, io);
  else
    hipLaunchKernelGGL((k_igemm<T, WM, WN, TM, TN, false>), grid, dim3(kThreads), 0, st, g, io);
  return hipGetLastError();
}

template <typename T, int WM, int WN, int TM, int TN>
hipError_t run_wgrad(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  dim3 grid((g.K + BN - 1) / BN, (g.N + BM - 1) / BM, replicas * io.splits);
  if constexpr (sizeof(T) == 4) {
    if (io.with_bias) {
      hipLaunchKernelGGL((k_wgrad<T, WM, WN, TM, TN, true>), grid, dim3(kThreads), 0, st, g, io);
      return hipGetLastError();
    }
  }
  hipLaunchKernelGGL((k_wgrad<T, WM, WN, TM, TN>), grid, dim3(kThreads), 0, st, g, io);
  return hipGetLastError();
}

// Output-channel tile of the bf16 kernels by layer width.
int bf16_ntile(int n) {
  if (n <= 32) return 32;
  if (n <= 64) return 64;
  if (n % 96 == 0 || n <= 96) return 96;
  return 128;
}

}  // namespace

hipError_t launch_igemm(hipStream_t st, int dtype, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io_in,
                        int *stat_splits) {
  if (g.M < 1 || g.N < 1 || g.K < 1 || replicas < 1 || replicas > 65535) return hipErrorInvalidValue;
  if (stat_splits) *stat_splits = 0;
  if (io_in.stat && stat_splits) {
    // the same order of choices as below, for the kernels whose epilogue can take the sums
    int S = 0;
    const bool smallk = conv_smallk_applicable(dtype, g, io_in);
    const bool halo = !smallk && conv_halo_applicable(dtype, g, io_in, out_f32);
    const bool fast = !smallk && !halo && !dgrad_s2_applicable(dtype, g, io_in, out_f32) &&
                      !gemm_ksplit_applicable(dtype, replicas, g, io_in) && igemm_fast_applicable(dtype, g, io_in);
    if (smallk) S = conv_smallk_stat_splits(g, out_f32);
    if (halo) S = conv_halo_stat_splits(g, replicas);
    if (fast) S = igemm_fast_stat_splits(dtype, out_f32, g, io_in);
    if (S > 0 && S <= io_in.stat_capacity) {
      *stat_splits = S;
      if (smallk) return launch_conv_smallk(st, dtype, out_f32, replicas, g, io_in);
      if (halo) return launch_conv_halo(st, replicas, g, io_in);
      return launch_igemm_fast(st, dtype, out_f32, replicas, g, io_in);
    }
  }
  GemmIO io = io_in;
  io.stat = nullptr;
  if (io.in_f32 && !(dtype == 1 && !out_f32 && conv_smallk_applicable(dtype, g, io))) return hipErrorInvalidValue;
  if (conv_smallk_applicable(dtype, g, io)) return launch_conv_smallk(st, dtype, out_f32, replicas, g, io);
  if (conv_halo_applicable(dtype, g, io, out_f32)) return launch_conv_halo(st, replicas, g, io);
  if (dgrad_s2_applicable(dtype, g, io, out_f32)) return launch_dgrad_s2(st, replicas, g, io);
  if (gemm_ksplit_applicable(dtype, replicas, g, io)) return launch_gemm_ksplit(st, dtype, out_f32, replicas, g, io);
  if (igemm_fast_applicable(dtype, g, io)) return launch_igemm_fast(st, dtype, out_f32, replicas, g, io);
  if (dtype == 0) return run_igemm<float, 2, 2, 1, 1>(st, out_f32, replicas, g, io);
  switch (bf16_ntile(g.N)) {
    case 32: return run_igemm<bf16_t, 4, 1, 1, 1>(st, out_f32, replicas, g, io);
    case 64: return run_igemm<bf16_t, 4, 1, 1, 2>(st, out_f32, replicas, g, io);
    case 96: return run_igemm<bf16_t, 4, 1, 1, 3>(st, out_f32, replicas, g, io);
    default: return run_igemm<bf16_t, 2, 2, 2, 2>(st, out_f32, replicas, g, io);
  }
}

hipError_t launch_wgrad(hipStream_t st, int dtype, int replicas, const ConvGeom &g, const WgradIO &io) {
  if (g.M < 1 || g.N < 1 || g.K < 1 || replicas < 1 || io.splits < 1 || (long long)replicas * io.splits > 65535 ||
      io.chunk < 32 || (io.chunk & 31))
    return hipErrorInvalidValue;
  if (wgrad_smallk_applicable(dtype, g) && aligned_to(io.dy, 16)) return launch_wgrad_smallk(st, replicas, g, io);
  if (io.x_f32) return hipErrorInvalidValue;  // only the kernel above reads fp32 memory for a bf16 layer
  if (wgrad_small_f32_applicable(dtype, g)) return launch_wgrad_small_f32(st, replicas, g, io);
  if (wgrad_window_applicable(dtype, g)) return launch_wgrad_window(st, replicas, g, io);
  if (wgrad9_applicable(dtype, g) && io.pairA && io.pairB) return launch_wgrad9(st, replicas, g, io);
  if (wgrad_fast_applicable(dtype, g) && io.pairA && io.pairB) return launch_wgrad_fast(st, replicas, g, io);
  if (dtype == 0) return run_wgrad<float, 2, 2, 1, 1>(st, replicas, g, io);
  switch (bf16_ntile(g.N)) {
    case 32: return run_wgrad<bf16_t, 1, 4, 1, 1>(st, replicas, g, io);
    case 64: return run_wgrad<bf16_t, 1, 4, 2, 1>(st, replicas, g, io);
    case 96: return run_wgrad<bf16_t, 1, 4, 3, 1>(st, replicas, g, io);
    default: return run_wgrad<bf16_t, 2, 2, 2, 2>(st, replicas, g, io);
  }
}

// mirrors the order of launch_wgrad
bool wgrad_takes_bias(int dtype, const ConvGeom &g, const WgradIO &io) {
  if (wgrad_smallk_applicable(dtype, g) && aligned_to(io.dy, 16)) return g.K < 32;
  if (wgrad_small_f32_applicable(dtype, g)) return g.K < 32;
  if (wgrad_window_applicable(dtype, g)) return false;
  if (dtype == 0) return true;  // the generic fp32 kernel
  return (wgrad9_applicable(dtype, g) || wgrad_fast_applicable(dtype, g)) && io.pairA && io.pairB;
}

int wgrad_plan(int dtype, int replicas, const ConvGeom &g, int *chunk_out) {
  if (wgrad9_applicable(dtype, g)) return wgrad9_plan(replicas, g, chunk_out);
  if (!wgrad_smallk_applicable(dtype, g) && !wgrad_small_f32_applicable(dtype, g) && wgrad_window_applicable(dtype, g))
    return wgrad_window_plan(replicas, g, chunk_out);
  int bm, bn;
  if (wgrad_smallk_applicable(dtype, g)) {
    bm = 128, bn = 32;
  } else if (wgrad_small_f32_applicable(dtype, g)) {
    bm = 32, bn = 32;  // one tile per replica
  } else if (wgrad_fast_applicable(dtype, g)) {
    wgrad_fast_tile(g, &bm, &bn);
  } else if (dtype == 0) {
    bm = 64, bn = 64;
  } else {
    bm = bf16_ntile(g.N);
    bn = 128;
  }
  const long long tiles = (long long)((g.K + bn - 1) / bn) * ((g.N + bm - 1) / bm) * replicas;
  const int steps = (g.M + 31) / 32;                  // contraction steps of 32 rows available
  static const int target = [] {
    const char *e = getenv("PARLE_WGRAD_BLOCKS");
    const int v = e ? atoi(e) : 0;
    return v > 0 ? v : 512;
  }();
  // at most `target` workgroups: two per compute unit, never a few stragglers in a third round
  // (the one-tile fp32 kernel is bound by the round trips of its operand loads, has few registers and writes a
  // 32 x 32 tile per split: it takes more, smaller splits)
  static const int target_small = [] {
    const char *e = getenv("PARLE_WGRAD_SMALL_BLOCKS");
    const int v = e ? atoi(e) : 0;
    return v > 0 ? v : 1024;
  }();
  const bool small_f32 = !wgrad_smallk_applicable(dtype, g) && wgrad_small_f32_applicable(dtype, g);
  long long want = (small_f32 ? target_small : target) / tiles;
  if (want > steps / 4) want = steps / 4;             // keep >= 4 steps (128 rows) per split
  if (want < 1) want = 1;
  const long long cap = 65535 / replicas;
  if (want > cap) want = cap;
  int chunk = (int)(((steps + want - 1) / want) * 32);
  int splits = (g.M + chunk - 1) / chunk;
  if (chunk_out) *chunk_out = chunk;
  return splits;
}
