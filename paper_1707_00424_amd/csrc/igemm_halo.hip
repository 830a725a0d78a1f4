// Stride-1 "same" convolutions (forward, and backward-data of such a layer) with the input patch
// staged ONCE in LDS and reused by every window tap.
//
// Why: the vector memory path of a CU delivers 64 bytes per clock; an implicit GEMM that fetches a
// fresh 256 x 32 operand tile from L1/L2 for each of the R*S taps moves (BM + BN) * 64 bytes per
// contraction step through that path, which caps the MFMA units near half of their rate for
// BN <= 128.  Here a workgroup owns 256 consecutive output pixels (whole image rows), loads the
// (rows + R - 1) x (width + S - 1) halo patch of 32 input channels once per channel chunk, and the
// MFMA fragments of all R*S taps are read from that patch at a tap-dependent LDS offset.  Global
// traffic per step drops to the weight tile plus 1/(R*S) of the patch.
//
// Step order: channel chunk outer, tap inner (the contraction order is free).  The weight tile of
// each step is double-buffered in LDS with a two-step register prefetch; the next chunk's patch
// is prefetched into registers during the R*S steps of the current one.
#include "igemm_dev.h"

namespace {

using namespace igemm_dev;

constexpr uint32_t kOob = 0x80000000u;
constexpr int kHaloSlots = 400;  // LDS patch capacity in pixels (32 KB at 32 channels + padding)

struct HaloGeom {
  int TH;          // output rows of one image inside a tile
  int nimg;        // images per tile (> 1 when an image has fewer than 256 pixels)
  int HR, HC;      // patch rows / columns per image = TH + R - 1, Q + S - 1
  int slots;       // nimg * HR * HC
  int omin_h, omin_w;  // smallest tap offset (input row = output row + offset)
};

template <int TN>
__global__ __launch_bounds__(kThreads) void k_conv_halo(const ConvGeom g, const GemmIO io, const HaloGeom hg) {
  typedef bf16_t T;
  constexpr int VW = 8, BK = 32, LK = BK + VW;
  constexpr int TM = 2, BM = 256, BN = TN * 32;  // four wavefronts stacked along the pixel axis
  constexpr int B_IT = (BN + 63) / 64;
  constexpr int H_IT = (kHaloSlots * 4 + kThreads - 1) / kThreads;
  // patch + double-buffered weight tiles; the epilogue reuses the same LDS as its staging strips
  constexpr int kPipeBytes = (kHaloSlots + 2 * BN) * LK * (int)sizeof(T);
  constexpr int kStageBytes = 4 * kStageFloats<TN> * (int)sizeof(float);
  __shared__ __attribute__((aligned(16))) char smem[kPipeBytes > kStageBytes ? kPipeBytes : kStageBytes];
  T *Hs = reinterpret_cast<T *>(smem);
  T(*Bs)[BN * LK] = reinterpret_cast<T(*)[BN * LK]>(smem + kHaloSlots * LK * sizeof(T));

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = blockIdx.z;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int lrow = tid >> 2, lkv = tid & 3;
  const int PQ = g.P * g.Q;
  const int RS = g.R * g.S;
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.in + rep * io.in_rs), 0, (int)(io.in_bytes), 0x00020000);
  const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.w + rep * io.w_rs), 0, (int)((long long)g.N * g.K * sizeof(T)), 0x00020000);

  // patch loader: vector v = it*256 + tid covers patch pixel v/4, channels 8*(v%4) .. +7 of the chunk
  const int b0 = m0 / PQ, p0 = (m0 % PQ) / g.Q;
  uint32_t h_off[H_IT];
#pragma unroll
  for (int it = 0; it < H_IT; ++it) {
    const int v = it * kThreads + tid, slot = v >> 2;
    uint32_t off = kOob;
    if (slot < hg.slots) {
      const int img = slot / (hg.HR * hg.HC), rem = slot % (hg.HR * hg.HC);
      const int hh = rem / hg.HC, ww = rem % hg.HC;
      const int b = b0 + img, ih = p0 + hh + hg.omin_h, iw = ww + hg.omin_w;
      if ((b * PQ < g.M) && ih >= 0 && ih < g.Hin && iw >= 0 && iw < g.Win)
        off = (uint32_t)((((b * g.Hin + ih) * g.Win + iw) * g.Cc + (v & 3) * VW) * (int)sizeof(T));
    }
    h_off[it] = off;
  }
  uint32_t b_off[B_IT];
#pragma unroll
  for (int i = 0; i < B_IT; ++i) {
    const int row = i * 64 + lrow, nrow = n0 + row;
    b_off[i] = (row < BN && nrow < g.N) ? (uint32_t)((nrow * g.K + lkv * VW) * (int)sizeof(T)) : kOob;
  }
  // fragment rows of this lane: pixel -> patch slot of tap offset (0, 0)
  int a_lds[TM];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    const int ml = wave * (TM * 32) + tm * 32 + (lane & 31);
    const int img = ml / (hg.TH * g.Q), rem = ml % (hg.TH * g.Q);
    const int ph = rem / g.Q, pw = rem % g.Q;
    a_lds[tm] = (((img * hg.HR + ph) * hg.HC + pw) * LK + (lane >> 5) * VW);
  }
  const int b_lds = (lane & 31) * LK + (lane >> 5) * VW;

  u4 hreg[H_IT];
  auto load_halo = [&](int chunk) {
    const uint32_t cb = (uint32_t)(chunk * BK * (int)sizeof(T));
    const bool live = chunk * BK < g.Cc;
#pragma unroll
    for (int it = 0; it < H_IT; ++it)
      hreg[it] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (live && h_off[it] != kOob) ? h_off[it] + cb : kOob, 0, 0);
  };
  auto store_halo = [&]() {
#pragma unroll
    for (int it = 0; it < H_IT; ++it) {
      const int v = it * kThreads + tid;
      if (v < kHaloSlots * 4) *(u4 *)&Hs[(v >> 2) * LK + (v & 3) * VW] = hreg[it];
    }
  };
  // weight tile of step t: channels of chunk t / RS at tap t % RS
  int ld_chunk = 0, ld_tap = 0, ld_t = 0;
  const int KT = (g.Cc / BK) * RS;
  auto load_b = [&](u4 (&breg)[B_IT]) {
    const uint32_t kb = (uint32_t)((ld_tap * g.Cc + ld_chunk * BK) * (int)sizeof(T));
    const bool live = ld_t < KT;
#pragma unroll
    for (int i = 0; i < B_IT; ++i)
      breg[i] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, (live && b_off[i] != kOob) ? b_off[i] + kb : kOob, 0, 0);
    ++ld_t;
    if (++ld_tap == RS) {
      ld_tap = 0;
      ++ld_chunk;
    }
  };
  auto store_b = [&](int buf, const u4 (&breg)[B_IT]) {
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

  // tap shift inside the patch: rows advance with r for a forward conv (sr = +1), against it for
  // backward-data (sr = -1); same for columns
  int tap_r = 0, tap_s = 0, chunk = 0;
  auto mma_step = [&](int buf) {
    const int dh = g.sr > 0 ? tap_r : g.R - 1 - tap_r, dw = g.sr > 0 ? tap_s : g.S - 1 - tap_s;
    const int shift = (dh * hg.HC + dw) * LK;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      u4 af[TM], bf[TN];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) af[tm] = *(const u4 *)&Hs[a_lds[tm] + shift + sub * 2 * VW];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) bf[tn] = *(const u4 *)&Bs[buf][tn * 32 * LK + b_lds + sub * 2 * VW];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) mma<T>(bf[tn], af[tm], acc[tm][tn]);
    }
  };
  // after the MFMAs of a step: move to the next tap; at the end of a chunk swap in the next patch
  auto next_tap = [&]() {
    if (++tap_s == g.S) {
      tap_s = 0;
      if (++tap_r == g.R) {
        tap_r = 0;
        ++chunk;
        __syncthreads();   // every wavefront is done reading the patch
        store_halo();
        load_halo(chunk + 1);
      }
    }
  };

  u4 b0r[B_IT], b1r[B_IT];
  load_halo(0);
  load_b(b0r);
  load_b(b1r);
  store_halo();
  load_halo(1);
  store_b(0, b0r);
  __syncthreads();
  int kt = 0;
  for (; kt + 1 < KT; kt += 2) {
    load_b(b0r);
    mma_step(0);
    store_b(1, b1r);
    next_tap();
    __syncthreads();
    load_b(b1r);
    mma_step(1);
    store_b(0, b0r);
    next_tap();
    __syncthreads();
  }
  if (kt < KT) mma_step(0);
  __syncthreads();  // patch and weight tiles are dead: their LDS becomes the staging strips
  store_tile_lds<T, TM, TN, false>(g, io, rep, m0 + wave * TM * 32, n0, lane, acc,
                                   reinterpret_cast<float *>(smem) + wave * kStageFloats<TN>);
}

template <int TN>
hipError_t run_halo(hipStream_t st, int replicas, const ConvGeom &g, const GemmIO &io, const HaloGeom &hg) {
  dim3 grid((g.M + 255) / 256, (g.N + TN * 32 - 1) / (TN * 32), replicas);
  hipLaunchKernelGGL((k_conv_halo<TN>), grid, dim3(kThreads), 0, st, g, io, hg);
  return hipGetLastError();
}

bool make_halo_geom(const ConvGeom &g, HaloGeom &hg) {
  const int BM = 256;
  if (g.sp != 1 || g.dshift != 0 || g.P != g.Hin || g.Q != g.Win) return false;
  if (BM % g.Q != 0) return false;
  const int PQ = g.P * g.Q;
  if (PQ >= BM) {
    if (PQ % BM != 0) return false;
    hg.TH = BM / g.Q, hg.nimg = 1;
  } else {
    if (BM % PQ != 0) return false;
    hg.TH = g.P, hg.nimg = BM / PQ;
  }
  hg.HR = hg.TH + g.R - 1, hg.HC = g.Q + g.S - 1;
  hg.slots = hg.nimg * hg.HR * hg.HC;
  const int o_first = g.off, o_last = g.off + (g.R - 1) * g.sr;
  hg.omin_h = o_first < o_last ? o_first : o_last;
  const int w_first = g.off, w_last = g.off + (g.S - 1) * g.sr;
  hg.omin_w = w_first < w_last ? w_first : w_last;
  return hg.slots <= kHaloSlots;
}

}  // namespace

bool conv_halo_applicable(int dtype, const ConvGeom &g, const GemmIO &io, bool out_f32) {
  HaloGeom hg;
  return dtype == 1 && !out_f32 && io.vecA && io.vecB && g.R * g.S > 1 && g.Cc % 32 == 0 && g.N % 4 == 0 &&
         io.ldc % 4 == 0 && io.in_bytes > 0 && io.in_bytes < (1LL << 31) && (long long)g.M * io.ldc * 4 < (1LL << 31) && (long long)g.N * g.K * 2 < (1LL << 31) &&
         g.M >= 256 && make_halo_geom(g, hg);
}

hipError_t launch_conv_halo(hipStream_t st, int replicas, const ConvGeom &g, const GemmIO &io) {
  HaloGeom hg;
  if (!make_halo_geom(g, hg)) return hipErrorInvalidValue;
  const int n = g.N;
  if (n <= 64) return run_halo<2>(st, replicas, g, io, hg);
  if (n <= 96 || n % 96 == 0) return run_halo<3>(st, replicas, g, io, hg);
  return run_halo<4>(st, replicas, g, io, hg);
}
