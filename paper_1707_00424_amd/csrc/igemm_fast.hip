// Vector fast paths of the implicit-GEMM kernels (channel counts that are multiples of the 16-byte
// vector width): the same tiling and MFMA layout as igemm.hip, with
//   * forward / backward-data: per-row validity of every tap precomputed as two bit masks (rows of the
//     window, columns of the window) and a linear tap offset, so a contraction step costs a few
//     integer instructions per 16-byte load instead of two range/parity tests and a multiply chain;
//     wavefront tiles up to 64x128 so that LDS fragment reads per MFMA drop below one;
//   * backward-weight (bf16): both operands are staged in LDS exactly as they lie in memory
//     ([pixel][channel], 16-byte loads and stores) and the MFMA fragments, which need the pixel index
//     contiguous, are fetched with the LDS transpose read (ds_read_b64_tr_b16).  Lane l of a 16-lane
//     group addresses row k0 + l/4, columns c0 + 4*(l%4) .. +3 and receives T[k0+e][c0+l], e = 0..3
//     (layout confirmed with an in-bounds probe on the device).
#include "igemm_dev.h"

namespace {

using namespace igemm_dev;
typedef short s4v __attribute__((ext_vector_type(4)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

template <int BYTES>
struct GatherVec;
template <>
struct GatherVec<16> {
  typedef u4 type;
  static __device__ __forceinline__ u4 zero() { return u4{0u, 0u, 0u, 0u}; }
};
template <>
struct GatherVec<8> {
  typedef u2 type;
  static __device__ __forceinline__ u2 zero() { return u2{0u, 0u}; }
};

// ---------------------------------------------------------------------------------------------
// forward / backward-data, vector path
// ---------------------------------------------------------------------------------------------
// GB: bytes per gather (16, or 8 for channel counts that are only a multiple of half a vector, e.g. 50 fp32
// channels); the LDS layout and the fragment reads are the same for both.
template <typename T, int WAVES_M, int WAVES_N, int TM, int TN, bool OUT_F32, int GB>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(TM * TN >= 8 ? 2 : 1))) void k_igemm_v(
    const ConvGeom g, const GemmIO io) {
  constexpr int VW = 16 / sizeof(T);   // elements per fragment read
  constexpr int GV = GB / sizeof(T);   // elements per gather
  constexpr int BK = 4 * VW;
  constexpr int LK = BK + VW;
  constexpr int LPR = BK / GV;         // lanes that share a tile row
  constexpr int RPP = kThreads / LPR;  // tile rows per pass
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  static_assert(BM % 64 == 0, "row tile must be a multiple of 64");
  constexpr int A_IT = BM / RPP, B_IT = (BN + RPP - 1) / RPP;
  typedef typename GatherVec<GB>::type gvec;
  __shared__ __attribute__((aligned(16))) T As[2][BM * LK];
  __shared__ __attribute__((aligned(16))) T Bs[2][BN * LK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int rep = blockIdx.z;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const T *__restrict__ in = (const T *)io.in + rep * io.in_rs;
  const T *__restrict__ w = (const T *)io.w + rep * io.w_rs;
  const int lrow = tid / LPR, lkv = tid % LPR;
  const int PQ = g.P * g.Q;

  int a_base[A_IT];
  uint32_t a_hmask[A_IT], a_wmask[A_IT];
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int m = m0 + i * RPP + lrow;
    const bool ok = m < g.M;
    const uint32_t mm = ok ? m : 0;
    const int b = fdiv(mm, g.dPQ), rem = mm - b * PQ;
    const int p = fdiv(rem, g.dQ), q = rem - p * g.Q;
    const int bh = p * g.sp + g.off, bw = q * g.sp + g.off;
    uint32_t hm = 0, wmk = 0;
    for (int r = 0; r < g.R; ++r) {
      int idx;
      hm |= (uint32_t)(ok && tap(bh + r * g.sr, g.dshift, g.Hin, idx)) << r;
    }
    for (int s = 0; s < g.S; ++s) {
      int idx;
      wmk |= (uint32_t)tap(bw + s * g.sr, g.dshift, g.Win, idx) << s;
    }
    a_hmask[i] = hm, a_wmask[i] = wmk;
    a_base[i] = (b * g.Hin + (bh >> g.dshift)) * g.Win * g.Cc + (bw >> g.dshift) * g.Cc;
  }
  int b_row[B_IT];
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    const int row = i * RPP + lrow, nrow = n0 + row;
    b_row[i] = (row < BN && nrow < g.N) ? nrow * g.K : -1;
  }
  int kk = lkv * GV, kr, ks, kc;
  {
    const uint32_t rs = fdiv(kk, g.dCc);
    kc = kk - rs * g.Cc;
    kr = fdiv(rs, g.dS);
    ks = rs - kr * g.S;
  }

  const gvec zero4 = GatherVec<GB>::zero();

  // Loads of steps past the end are fully masked (tap row index beyond the window, kk >= K), so
  // the pipeline below may always run two steps ahead without touching memory out of range.
  auto load_tiles = [&](gvec (&areg)[A_IT], gvec (&breg)[B_IT]) {
    const int toff = g.sr * (((kr >> g.dshift) * g.Win + (ks >> g.dshift)) * g.Cc) + kc;
    const int krs = kr < 31 ? kr : 31;
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const bool ok = ((a_hmask[i] >> krs) & (a_wmask[i] >> ks) & 1u) != 0;
      areg[i] = ok ? *(const gvec *)(in + a_base[i] + toff) : zero4;
    }
    const bool kok = kk < g.K;
#pragma unroll
    for (int i = 0; i < B_IT; ++i) breg[i] = (kok && b_row[i] >= 0) ? *(const gvec *)(w + b_row[i] + kk) : zero4;
  };
  // branch-free: Cc >= VW (applicability test), so one step of BK = 4*VW crosses at most four tap boundaries
  auto advance_k = [&]() {
    kk += BK;
    kc += BK;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const bool wrap = kc >= g.Cc;
      kc -= wrap ? g.Cc : 0;
      ks += wrap ? 1 : 0;
      const bool wrap_s = ks == g.S;
      ks = wrap_s ? 0 : ks;
      kr += wrap_s ? 1 : 0;
    }
  };
  auto store_tiles = [&](int buf, const gvec (&areg)[A_IT], const gvec (&breg)[B_IT]) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) *(gvec *)&As[buf][(i * RPP + lrow) * LK + lkv * GV] = areg[i];
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int row = i * RPP + lrow;
      if (BN % RPP == 0 || row < BN) *(gvec *)&Bs[buf][row * LK + lkv * GV] = breg[i];
    }
  };

  f16v acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

  // Software pipeline, two steps deep: global loads of step t+2 are issued before the MFMAs of
  // step t, the registers of step t+1 go to the other LDS buffer after them, one barrier per step.
  // Two register sets, so the loop is unrolled by two; the body has no data-dependent branches.
  const int KT = (g.K + BK - 1) / BK;
  gvec a0[A_IT], b0[B_IT], a1[A_IT], b1[B_IT];
  load_tiles(a0, b0);
  advance_k();
  load_tiles(a1, b1);
  store_tiles(0, a0, b0);
  __syncthreads();
  int kt = 0;
  for (; kt + 1 < KT; kt += 2) {
    advance_k();
    load_tiles(a0, b0);
    mma_tile<T, TM, TN, LK, VW>(As[0], Bs[0], wm * TM * 32, wn * TN * 32, lane, acc);
    store_tiles(1, a1, b1);
    __syncthreads();
    advance_k();
    load_tiles(a1, b1);
    mma_tile<T, TM, TN, LK, VW>(As[1], Bs[1], wm * TM * 32, wn * TN * 32, lane, acc);
    store_tiles(0, a0, b0);
    __syncthreads();
  }
  if (kt < KT) mma_tile<T, TM, TN, LK, VW>(As[0], Bs[0], wm * TM * 32, wn * TN * 32, lane, acc);
  store_tile<T, TM, TN, OUT_F32>(g, io, rep, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, acc);
}


// ---------------------------------------------------------------------------------------------
// forward / backward-data, uniform-tap path: the channel count is a multiple of the contraction
// step (Cc % BK == 0), so a whole step lies inside one window tap and the tap bookkeeping is
// wavefront-uniform (scalar registers).  Operands are fetched with raw buffer loads: a lane whose
// tap falls outside the image, or whose row is beyond the tensor, gets an offset past the buffer's
// range and the hardware returns zeros -- no branch, no select.  Accumulator tiles are kept
// transposed so the epilogue writes four consecutive channels per lane.
// ---------------------------------------------------------------------------------------------
constexpr uint32_t kOob = 0x80000000u;  // beyond any per-replica tensor (each is < 2 GiB)

// STAT: also the column sums of the output for the batch-norm behind the layer (see store_tile_lds), one partial
// row per row tile.
// (register budgets: the widest tiles are held to two wavefronts per SIMD - left alone, their epilogue variants take
// more than 256 registers and a compute unit then holds one workgroup - and the 128 x 64 and 128 x 128 tiles, which
// came out a few registers above 168, to three)
template <typename T, int WAVES_M, int WAVES_N, int TM, int TN, bool OUT_F32, bool STAT = false>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(TM * TN >= 8 ? 2 : (TM * TN == 2 || (TM * TN == 4 && WAVES_M == 2) ? 3 : 1)))) void k_igemm_u(
    const ConvGeom g, const GemmIO io) {
  constexpr int VW = 16 / sizeof(T);
  constexpr int BK = 4 * VW;
  constexpr int LK = BK + VW;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  static_assert(BM % 64 == 0, "row tile must be a multiple of 64");
  constexpr int A_IT = BM / 64, B_IT = (BN + 63) / 64;
  // operand tiles (double-buffered); the epilogue reuses the same LDS as its staging strips
  constexpr int kPipeBytes = 2 * (BM + BN) * LK * (int)sizeof(T);
  constexpr int kStageBytes = (4 * kStageFloats<TN> + (STAT ? WAVES_M * 2 * BN : 0)) * (int)sizeof(float);
  __shared__ __attribute__((aligned(16))) char smem[kPipeBytes > kStageBytes ? kPipeBytes : kStageBytes];
  T(*As)[BM * LK] = reinterpret_cast<T(*)[BM * LK]>(smem);
  T(*Bs)[BN * LK] = reinterpret_cast<T(*)[BN * LK]>(smem + 2 * BM * LK * sizeof(T));

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int rep = blockIdx.z;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int lrow = tid >> 2, lkv = tid & 3;
  const int PQ = g.P * g.Q;
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.in + rep * io.in_rs), 0, (int)(io.in_bytes), 0x00020000);
  const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.w + rep * io.w_rs), 0, (int)((long long)g.N * g.K * sizeof(T)), 0x00020000);

  // per row: byte offset of its window origin (+ this lane's vector inside a step) and one validity
  // bit per tap
  __shared__ uint32_t taps_any;
  if (tid == 0) taps_any = 0;
  __syncthreads();
  uint32_t a_off[A_IT], a_taps[A_IT], my_taps = 0;
#pragma unroll
  for (int i = 0; i < A_IT; ++i) {
    const int m = m0 + i * 64 + lrow;
    const bool ok = m < g.M;
    const uint32_t mm = ok ? row_pixel(g, (uint32_t)m) : 0;
    const int b = fdiv(mm, g.dPQ), rem = mm - b * PQ;
    const int p = fdiv(rem, g.dQ), q = rem - p * g.Q;
    const int bh = p * g.sp + g.off, bw = q * g.sp + g.off;
    // window columns the row can reach, then one copy of that mask per reachable window row
    uint32_t wmask = 0, taps = 0;
    int idx;
    for (int s2 = 0; s2 < g.S; ++s2) wmask |= (uint32_t)tap(bw + s2 * g.sr, g.dshift, g.Win, idx) << s2;
    for (int r = 0; r < g.R; ++r) taps |= tap(bh + r * g.sr, g.dshift, g.Hin, idx) ? wmask << (r * g.S) : 0u;
    taps = ok ? taps : 0u;
    a_taps[i] = taps;
    my_taps |= taps;
    a_off[i] = (uint32_t)(((b * g.Hin + (bh >> g.dshift)) * g.Win * g.Cc + (bw >> g.dshift) * g.Cc + lkv * VW) * (int)sizeof(T));
  }
  uint32_t b_off[B_IT];
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    const int row = i * 64 + lrow, nrow = n0 + row;
    b_off[i] = (row < BN && nrow < g.N) ? (uint32_t)((nrow * g.K + lkv * VW) * (int)sizeof(T)) : kOob;
  }
  // taps that no row of this tile can reach are skipped altogether (stride-2 backward-data with
  // parity-class row order: a tile reaches 1, 2 or 4 of 9 taps)
  if (my_taps) atomicOr(&taps_any, my_taps);
  __syncthreads();
  const uint32_t tile_taps = __builtin_amdgcn_readfirstlane(taps_any);
  const int KT = __builtin_popcount(tile_taps) * (g.Cc / BK);
  // wavefront-uniform contraction state: tap index, first channel kc of the step, steps loaded
  int tapi = tile_taps ? __builtin_ctz(tile_taps) : 0, kc = 0, kt_load = 0;

  auto load_tiles = [&](u4 (&areg)[A_IT], u4 (&breg)[B_IT]) {
    const int kr = (int)fdiv((uint32_t)tapi, g.dS), ks = tapi - kr * g.S;
    const uint32_t toff = (uint32_t)((g.sr * (((kr >> g.dshift) * g.Win + (ks >> g.dshift)) * g.Cc) + kc) * (int)sizeof(T));
    const bool live = kt_load < KT;  // steps past the end load nothing
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const bool ok = live && ((a_taps[i] >> tapi) & 1u);
      areg[i] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, ok ? a_off[i] + toff : kOob, 0, 0);
    }
    const uint32_t kb = (uint32_t)((tapi * g.Cc + kc) * (int)sizeof(T));
#pragma unroll
    for (int i = 0; i < B_IT; ++i)
      breg[i] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, (live && b_off[i] != kOob) ? b_off[i] + kb : kOob, 0, 0);
  };
  auto advance_k = [&]() {
    ++kt_load;
    kc += BK;
    if (kc >= g.Cc) {
      kc = 0;
      const uint32_t rest = tile_taps & ~((2u << tapi) - 1u);
      tapi = rest ? __builtin_ctz(rest) : 0;
    }
  };
  auto store_tiles = [&](int buf, const u4 (&areg)[A_IT], const u4 (&breg)[B_IT]) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) *(u4 *)&As[buf][(i * 64 + lrow) * LK + lkv * VW] = areg[i];
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

  // Software pipeline: LDS is double-buffered, and D steps travel from memory in registers.  Memory answers in more
  // cycles than a step multiplies (a step is TM*TN*2 MFMAs per wavefront), so the tile stored to LDS in step t was
  // requested in step t - D + 1: with two register sets every step waited out most of a memory round trip.
  constexpr int D = (A_IT + B_IT) * TM * TN <= 24 ? 4 : 3;
  u4 ra[D][A_IT], rb[D][B_IT];
#pragma unroll
  for (int i = 0; i < D; ++i) {
    if (i) advance_k();
    load_tiles(ra[i], rb[i]);  // steps past the end load nothing
  }
  store_tiles(0, ra[0], rb[0]);
  __syncthreads();
  // step t: set `cur` held tile t (in LDS since the previous step) and is refilled with tile t + D; set `nxt`
  // holds tile t + 1, which goes to the other LDS buffer
  auto step = [&](int t, u4 (&ca)[A_IT], u4 (&cb)[B_IT], const u4 (&na)[A_IT], const u4 (&nb)[B_IT]) {
    advance_k();
    load_tiles(ca, cb);
    mma_tile_t<T, TM, TN, LK, VW>(As[t & 1], Bs[t & 1], wm * TM * 32, wn * TN * 32, lane, acc);
    store_tiles((t + 1) & 1, na, nb);
    __syncthreads();
  };
  int kt = 0;
  for (; kt + D - 1 < KT; kt += D) {
#pragma unroll
    for (int i = 0; i < D; ++i) step(kt + i, ra[i], rb[i], ra[(i + 1) % D], rb[(i + 1) % D]);
  }
#pragma unroll
  for (int i = 0; i < D - 1; ++i)
    if (kt + i < KT) step(kt + i, ra[i], rb[i], ra[(i + 1) % D], rb[(i + 1) % D]);
  // the barrier that ended the last step: operand tiles are dead, their LDS becomes the staging strips
  // sums of wavefront (wm, wn): row wm of [WAVES_M][2][BN], columns wn * TN * 32 ...
  float *wsums = reinterpret_cast<float *>(smem) + 4 * kStageFloats<TN>;
  store_tile_lds<T, TM, TN, OUT_F32, STAT>(g, io, rep, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, acc,
                                           reinterpret_cast<float *>(smem) + wave * kStageFloats<TN>,
                                           wsums + wm * 2 * BN + wn * TN * 32, BN);
  if (STAT) write_tile_sums<BN, WAVES_M>(g, io, rep, gridDim.x, blockIdx.x, n0, tid, wsums);
}

// ---------------------------------------------------------------------------------------------
// backward-weight, bf16, LDS transpose reads.  out[n, k] = sum_m dy[m, n] * gather(m, k).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ u4 lds_tr_frag(const bf16_t *tile, int ld, int krow, int col) {
  // 8 contraction values (rows krow .. krow+7 as seen by this lane's 16-lane group) of column `col + l%16`
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

// BIAS: the workgroups of the first column tile also sum the dy vectors they stage and write the layer's bias
// gradient, the column sums of dy, behind the weights.
// (the 256 x 128 tile is held to two wavefronts per SIMD: at 264 registers a compute unit held one workgroup)
template <int WAVES_M, int WAVES_N, int TM, int TN, bool BIAS>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(TM * TN >= 8 ? 2 : 1))) void k_wgrad_tr(
    const ConvGeom g, const WgradIO io) {
  constexpr int BKM = 32;  // pixels per contraction step
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  constexpr int LDA = BM + 16, LDB = BN + 16;  // row strides = 32 (mod 128) bytes: conflict-free transpose reads
  constexpr int AV = BM / 8, BV = BN / 8;      // 16-byte vectors per pixel row
  static_assert(kThreads % BV == 0, "a thread must own one column vector of the gathered operand");
  constexpr int A_IT = (BKM * AV + kThreads - 1) / kThreads;
  constexpr int B_ROWS = kThreads / BV, B_IT = BKM / B_ROWS;
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BKM * LDA];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BKM * LDB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int rep = blockIdx.z / io.splits, split = blockIdx.z % io.splits;
  const int n0 = blockIdx.y * BM, k0 = blockIdx.x * BN;
  const bf16_t *__restrict__ dy = (const bf16_t *)io.dy + rep * io.dy_rs;
  const bf16_t *__restrict__ x = (const bf16_t *)io.x + rep * io.x_rs;
  const int m_begin = split * io.chunk, m_end = min(g.M, m_begin + io.chunk);
  const int PQ = g.P * g.Q;

  // gathered operand: this thread's fixed column vector (tap r, s and first channel)
  const int bcv = tid % BV, brow0 = tid / BV;
  const int kcol = k0 + bcv * 8;
  const bool bcol_ok = kcol < g.K;
  int b_r, b_s, b_c;
  {
    const uint32_t kk = bcol_ok ? kcol : 0;
    const uint32_t rs = fdiv(kk, g.dCc);
    b_c = kk - rs * g.Cc;
    b_r = fdiv(rs, g.dS);
    b_s = rs - b_r * g.S;
  }
  const int b_tapoff = ((b_r - (-g.off)) * g.Win + (b_s - (-g.off))) * g.Cc + b_c;  // (r - pad, s - pad)

  const u4 zero4 = {0u, 0u, 0u, 0u};
  const bool tally = BIAS && blockIdx.x == 0;
  float bsum[BIAS ? A_IT : 1][8];
  if (BIAS) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) bsum[i][e] = 0.f;
  }

  // rows at or beyond m_end are masked, so the pipeline may load two steps ahead unconditionally
  auto load_tiles = [&](int mbase, u4 (&areg)[A_IT], u4 (&breg)[B_IT]) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int v = i * kThreads + tid;
      const int row = v / AV, cv = v % AV;
      const int m = mbase + row, n = n0 + cv * 8;
      const bool ok = (BKM * AV % kThreads == 0 || v < BKM * AV) && m < m_end && n < g.N;
      areg[i] = ok ? *(const u4 *)(dy + (long long)m * g.N + n) : zero4;
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
      const int m = mbase + i * B_ROWS + brow0;
      const bool mok = m < m_end;
      const uint32_t mm = mok ? m : 0;
      const int b = fdiv(mm, g.dPQ), rem = mm - b * PQ;
      const int p = fdiv(rem, g.dQ), q = rem - p * g.Q;
      const int ih = p * g.sp + g.off + b_r, iw = q * g.sp + g.off + b_s;
      const bool ok = mok && bcol_ok && ih >= 0 && ih < g.Hin && iw >= 0 && iw < g.Win;
      const int base = ((b * g.Hin + p * g.sp) * g.Win + q * g.sp) * g.Cc;
      breg[i] = ok ? *(const u4 *)(x + base + b_tapoff) : zero4;
    }
  };
  auto store_tiles = [&](int buf, const u4 (&areg)[A_IT], const u4 (&breg)[B_IT]) {
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int v = i * kThreads + tid;
      if (BKM * AV % kThreads == 0 || v < BKM * AV) *(u4 *)&As[buf][(v / AV) * LDA + (v % AV) * 8] = areg[i];
    }
#pragma unroll
    for (int i = 0; i < B_IT; ++i) *(u4 *)&Bs[buf][(i * B_ROWS + brow0) * LDB + bcv * 8] = breg[i];
    if (BIAS && tally) {  // masked rows and columns hold zeros
#pragma unroll
      for (int i = 0; i < A_IT; ++i) {
        const uint32_t w[4] = {areg[i].x, areg[i].y, areg[i].z, areg[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          bsum[i][2 * e] += __uint_as_float(w[e] << 16);
          bsum[i][2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
        }
      }
    }
  };

  f16v acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

  // fragment addressing: 16-lane group gq covers columns 16*(gq%2) .. +15 and contraction half gq/2
  const int gq = lane >> 4, j = lane & 15;
  const int frag_k = 8 * (gq >> 1) + (j >> 2), frag_c = 16 * (gq & 1) + 4 * (j & 3);

  auto mma_step = [&](const bf16_t *at, const bf16_t *bt) {
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      u4 af[TM], bf[TN];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) af[tm] = lds_tr_frag(at, LDA, sub * 16 + frag_k, wm * TM * 32 + tm * 32 + frag_c);
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) bf[tn] = lds_tr_frag(bt, LDB, sub * 16 + frag_k, wn * TN * 32 + tn * 32 + frag_c);
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) mma<bf16_t>(af[tm], bf[tn], acc[tm][tn]);
    }
  };
  // two-step-deep software pipeline, unrolled by two (see k_igemm_v); an empty split writes zeros
  const int KT = m_end > m_begin ? (m_end - m_begin + BKM - 1) / BKM : 0;
  u4 a0[A_IT], b0[B_IT], a1[A_IT], b1[B_IT];
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
    // vector v of a step lies in pixel row v / AV: the 32 rows are added in a fixed order
    float *bs = (float *)&As[0][0];  // [BKM][BM]
    static_assert(sizeof(As) >= BKM * BM * 4, "bias staging");
    __syncthreads();  // the last fragments have been read
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
      const int v = i * kThreads + tid;
      if (BKM * AV % kThreads == 0 || v < BKM * AV) {
#pragma unroll
        for (int e = 0; e < 8; ++e) bs[(v / AV) * BM + (v % AV) * 8 + e] = bsum[i][e];
      }
    }
    __syncthreads();
    for (int c = tid; c < BM; c += kThreads) {
      float t = 0.f;
      for (int q = 0; q < BKM; ++q) t += bs[q * BM + c];
      if (n0 + c < g.N) out[(long long)g.N * g.K + n0 + c] = t;
    }
  }
}

template <typename T, int WM, int WN, int TM, int TN, int GB = 16>
hipError_t run_v(hipStream_t st, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  dim3 grid((g.M + BM - 1) / BM, (g.N + BN - 1) / BN, replicas);
  if (out_f32)
    hipLaunchKernelGGL((k_igemm_v<T, WM, WN, TM, TN, true, GB>), grid, dim3(kThreads), 0, st, g, io);
  else
    hipLaunchKernelGGL((k_igemm_v<T, WM, WN, TM, TN, false, GB>), grid, dim3(kThreads), 0, st, g, io);
  return hipGetLastError();
}

template <typename T, int WM, int WN, int TM, int TN>
hipError_t run_u(hipStream_t st, bool out_f32, int replicas, const ConvGeom &g, const GemmIO &io) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  dim3 grid((g.M + BM - 1) / BM, (g.N + BN - 1) / BN, replicas);
  constexpr bool kStat = sizeof(T) == 2 && WM == 2 && WN == 2 && TM == 2 && (TN == 2 || TN == 4);  // see igemm_fast_stat_splits
  if (io.stat) {
    if (!kStat || out_f32) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_igemm_u<T, WM, WN, TM, TN, false, kStat>), grid, dim3(kThreads), 0, st, g, io);
  } else if (out_f32) {
    hipLaunchKernelGGL((k_igemm_u<T, WM, WN, TM, TN, true>), grid, dim3(kThreads), 0, st, g, io);
  } else {
    hipLaunchKernelGGL((k_igemm_u<T, WM, WN, TM, TN, false>), grid, dim3(kThreads), 0, st, g, io);
  }
  return hipGetLastError();
}

template <int WM, int WN, int TM, int TN>
hipError_t run_tr(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io) {
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  dim3 grid((g.K + BN - 1) / BN, (g.N + BM - 1) / BM, replicas * io.splits);
  if (io.with_bias)
    hipLaunchKernelGGL((k_wgrad_tr<WM, WN, TM, TN, true>), grid, dim3(kThreads), 0, st, g, io);
  else
    hipLaunchKernelGGL((k_wgrad_tr<WM, WN, TM, TN, false>), grid, dim3(kThreads), 0, st, g, io);
  return hipGetLastError();
}

// tall (256-row) tiles only when they still leave enough workgroups to fill the chip
bool tall_ok(const ConvGeom &g, int bn, int replicas) {
  const long long blocks = (long long)((g.M + 255) / 256) * ((g.N + bn - 1) / bn) * replicas;
  return blocks >= 512;
}

}  // namespace

namespace {
bool full_vector_ok(int dtype, const ConvGeom &g, const GemmIO &io) {
  const int vw = dtype ? 8 : 4;
  return io.vecA && io.vecB && g.Cc % vw == 0 && g.K % vw == 0 && g.R <= 16 && g.S <= 16;
}
// fp32 channel counts that are even but no multiple of four (LeNet's 50): 8-byte gathers
bool half_vector_ok(int dtype, const ConvGeom &g, const GemmIO &io) {
  return dtype == 0 && g.Cc % 2 == 0 && g.Cc >= 4 && g.R <= 16 && g.S <= 16 && aligned_to(io.in, 8) &&
         io.in_rs % 2 == 0 && aligned_to(io.w, 8) && io.w_rs % 2 == 0;
}
}  // namespace

bool igemm_fast_applicable(int dtype, const ConvGeom &g, const GemmIO &io) {
  return full_vector_ok(dtype, g, io) || half_vector_ok(dtype, g, io);
}

// Uniform-tap kernel: a whole contraction step inside one tap, vector epilogue, 32-bit byte offsets.
bool uniform_ok(int dtype, const ConvGeom &g, const GemmIO &io) {
  const int bk = dtype ? 32 : 16;
  return g.Cc % bk == 0 && g.R * g.S <= 32 && g.N % 4 == 0 && io.ldc % 4 == 0 && io.in_bytes > 0 &&
         io.in_bytes < (1LL << 31) && (long long)g.M * io.ldc * 4 < (1LL << 31) && (long long)g.N * g.K * (dtype ? 2 : 4) < (1LL << 31);
}

// Partial rows of column sums a launch with io.stat set writes: one per 128 output rows, for the bf16 layers the
// uniform-tap kernel runs on 128 x 128 or 128 x 256 tiles (more than 96 output channels, not a multiple of 192);
// 0: none.  Mirrors the choice of launch_igemm_fast below.
int igemm_fast_stat_splits(int dtype, bool out_f32, const ConvGeom &g, const GemmIO &io) {
  if (dtype != 1 || out_f32 || !(full_vector_ok(dtype, g, io) && uniform_ok(dtype, g, io))) return 0;
  const int n = g.N;
  const bool t22 = n > 96 && n <= 128, t24 = n > 192 && n % 192 != 0;
  return t22 || t24 ? (g.M + 127) / 128 : 0;
}

hipError_t launch_igemm_fast(hipStream_t st, int dtype, bool out_f32, int replicas, const ConvGeom &g_in,
                             const GemmIO &io) {
  ConvGeom g = g_in;
  g.plp = g.plq = 0;
  if (full_vector_ok(dtype, g, io) && uniform_ok(dtype, g, io)) {
    // stride-2 backward data on power-of-two images: rows grouped by parity class
    auto log2_exact = [](int v) {
      int l = 0;
      while ((1 << l) < v) ++l;
      return (1 << l) == v ? l : 0;
    };
    if (g.dshift == 1 && log2_exact(g.P) >= 1 && log2_exact(g.Q) >= 1) g.plp = log2_exact(g.P), g.plq = log2_exact(g.Q);
    if (dtype == 0) return run_u<float, 2, 2, 1, 1>(st, out_f32, replicas, g, io);
    const int n = g.N;
    if (n <= 32) return run_u<bf16_t, 4, 1, 1, 1>(st, out_f32, replicas, g, io);
    if (n <= 64)
      return tall_ok(g, 64, replicas) ? run_u<bf16_t, 4, 1, 2, 2>(st, out_f32, replicas, g, io)
                                      : run_u<bf16_t, 4, 1, 1, 2>(st, out_f32, replicas, g, io);
    if (n <= 96)
      return tall_ok(g, 96, replicas) ? run_u<bf16_t, 4, 1, 2, 3>(st, out_f32, replicas, g, io)
                                      : run_u<bf16_t, 4, 1, 1, 3>(st, out_f32, replicas, g, io);
    if (n <= 128) return run_u<bf16_t, 2, 2, 2, 2>(st, out_f32, replicas, g, io);
    if (n <= 192 || n % 192 == 0) return run_u<bf16_t, 2, 2, 2, 3>(st, out_f32, replicas, g, io);
    return run_u<bf16_t, 2, 2, 2, 4>(st, out_f32, replicas, g, io);
  }
  if (dtype == 0) {
    if (!full_vector_ok(dtype, g, io))
      return g.N <= 32 ? run_v<float, 4, 1, 1, 1, 8>(st, out_f32, replicas, g, io)
                       : run_v<float, 2, 2, 1, 1, 8>(st, out_f32, replicas, g, io);
    return g.N <= 32 ? run_v<float, 4, 1, 1, 1>(st, out_f32, replicas, g, io)
                     : run_v<float, 2, 2, 1, 1>(st, out_f32, replicas, g, io);
  }
  const int n = g.N;
  if (n <= 32) return run_v<bf16_t, 4, 1, 1, 1>(st, out_f32, replicas, g, io);
  if (n <= 64)
    return tall_ok(g, 64, replicas) ? run_v<bf16_t, 4, 1, 2, 2>(st, out_f32, replicas, g, io)
                                    : run_v<bf16_t, 4, 1, 1, 2>(st, out_f32, replicas, g, io);
  if (n <= 96)
    return tall_ok(g, 96, replicas) ? run_v<bf16_t, 4, 1, 2, 3>(st, out_f32, replicas, g, io)
                                    : run_v<bf16_t, 4, 1, 1, 3>(st, out_f32, replicas, g, io);
  if (n <= 128) return run_v<bf16_t, 2, 2, 2, 2>(st, out_f32, replicas, g, io);
  if (n <= 192 || n % 192 == 0) return run_v<bf16_t, 2, 2, 2, 3>(st, out_f32, replicas, g, io);
  return run_v<bf16_t, 2, 2, 2, 4>(st, out_f32, replicas, g, io);
}

bool wgrad_fast_applicable(int dtype, const ConvGeom &g) {
  return dtype == 1 && g.Cc % 8 == 0 && g.N % 8 == 0 && g.N >= 32 && g.dshift == 0 && g.sr == 1;
}

void wgrad_fast_tile(const ConvGeom &g, int *bm, int *bn) {
  const int n = g.N;
  if (n <= 32) *bm = 32, *bn = 128;
  else if (n <= 64) *bm = 64, *bn = 256;
  else if (n <= 96) *bm = 96, *bn = 256;
  else if (n <= 128) *bm = 128, *bn = 128;
  else if (n <= 192 || n % 192 == 0) *bm = 192, *bn = 128;
  else *bm = 256, *bn = 128;
}

hipError_t launch_wgrad_fast(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io) {
  int bm, bn;
  wgrad_fast_tile(g, &bm, &bn);
  switch (bm) {
    case 32: return run_tr<1, 4, 1, 1>(st, replicas, g, io);
    case 64: return run_tr<1, 4, 2, 2>(st, replicas, g, io);
    case 96: return run_tr<1, 4, 3, 2>(st, replicas, g, io);
    case 128: return run_tr<2, 2, 2, 2>(st, replicas, g, io);
    case 192: return run_tr<2, 2, 3, 2>(st, replicas, g, io);
    default: return run_tr<2, 2, 4, 2>(st, replicas, g, io);
  }
}
