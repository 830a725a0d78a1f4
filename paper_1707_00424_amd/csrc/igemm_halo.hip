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
//
// Stride-2 3x3 layers (forward) run the same body on 128 output pixels per workgroup: their patch is
// (2 rows + 1) x (2 width + 1) input pixels, four times the output tile, and every input pixel is under some tap, so
// staging the patch once reads the input exactly once, in whole rows; a kernel that gathers the rows of each tap
// from memory reads 64-byte pieces 2 pixels apart, nine times over, and is bound by that.
#include <stdlib.h>

#include "igemm_dev.h"

namespace {

using namespace igemm_dev;

constexpr uint32_t kOob = 0x80000000u;
constexpr int kHaloSlots = 400;    // LDS patch capacity in pixels (32 KB at 32 channels + padding)
constexpr int kHaloSlotsS2 = 592;  // stride 2: 17 x 33 (16 output columns) or 2 x 17 x 17 (two 8 x 8 outputs), 47 KB

struct HaloGeom {
  int TH;          // output rows of one image inside a tile
  int nimg;        // images per tile (> 1 when an image has fewer than 256 pixels)
  int HR, HC;      // patch rows / columns per image = TH + R - 1, Q + S - 1
  int slots;       // nimg * HR * HC
  int omin_h, omin_w;  // smallest tap offset (input row = output row + offset)
  FastDiv dImg, dHC, dRows;  // by HR*HC, HC and TH*Q (no integer division on the device)
  int tiles, nb, bn;  // pixel tiles, column blocks and their width in channels (set with the grid)
};

// LDS of a workgroup with TN column tiles: patch + a ring of three weight tiles; the epilogue reuses the same
// bytes as its staging strips
// with STAT, the column sums of the four wavefronts (2 x TN*32 floats each) lie behind the strips
template <int TN, bool STAT = false, int SLOTS = kHaloSlots>
constexpr int halo_lds_bytes() {
  constexpr int pipe = (SLOTS + 3 * TN * 32) * (32 + 8) * 2;
  constexpr int stage = 4 * kStageFloats<TN> * (int)sizeof(float) + (STAT ? 4 * 2 * TN * 32 * (int)sizeof(float) : 0);
  return pipe > stage ? pipe : stage;
}

// `tile`, `col`: pixel tile and column block of this workgroup; column blocks before it are hg.bn wide.
// TM: 32-pixel tiles per wavefront (the workgroup's tile is TM * 128 output pixels); SLOTS: patch capacity; SP: stride.
template <int TN, bool STAT, int TM = 2, int SLOTS = kHaloSlots, int SP = 1>
__device__ __forceinline__ void conv_halo_body(const ConvGeom &g, const GemmIO &io, const HaloGeom &hg, char *smem,
                                               int tile, int col) {
  typedef bf16_t T;
  constexpr int VW = 8, BK = 32, LK = BK + VW;
  constexpr int BM = TM * 128, BN = TN * 32;  // four wavefronts stacked along the pixel axis
  constexpr int B_IT = (BN + 63) / 64;
  constexpr int H_IT = (SLOTS * 4 + kThreads - 1) / kThreads;
  T *Hs = reinterpret_cast<T *>(smem);
  T *Bs = reinterpret_cast<T *>(smem + SLOTS * LK * sizeof(T));  // tile i of the ring at Bs + i * BN * LK

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = blockIdx.z;
  const int m0 = tile * BM, n0 = col * hg.bn;
  const int lrow = tid >> 2, lkv = tid & 3;
  const int PQ = g.P * g.Q;
  const int RS = g.R * g.S;
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.in + rep * io.in_rs), 0, (int)(io.in_bytes), 0x00020000);
  const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.w + rep * io.w_rs), 0, (int)((long long)g.N * g.K * sizeof(T)), 0x00020000);

  // patch loader: vector v = it*256 + tid covers patch pixel v/4, channels 8*(v%4) .. +7 of the chunk
  const int b0 = (int)fdiv((uint32_t)m0, g.dPQ), p0 = (int)fdiv((uint32_t)(m0 - b0 * PQ), g.dQ);
  uint32_t h_off[H_IT];
#pragma unroll
  for (int it = 0; it < H_IT; ++it) {
    const int v = it * kThreads + tid, slot = v >> 2;
    uint32_t off = kOob;
    if (slot < hg.slots) {
      const int img = (int)fdiv((uint32_t)slot, hg.dImg), rem = slot - img * hg.HR * hg.HC;
      const int hh = (int)fdiv((uint32_t)rem, hg.dHC), ww = rem - hh * hg.HC;
      const int b = b0 + img, ih = SP * p0 + hh + hg.omin_h, iw = ww + hg.omin_w;
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
    const int img = (int)fdiv((uint32_t)ml, hg.dRows), rem = ml - img * hg.TH * g.Q;
    const int ph = (int)fdiv((uint32_t)rem, g.dQ), pw = rem - ph * g.Q;
    a_lds[tm] = (((img * hg.HR + SP * ph) * hg.HC + SP * pw) * LK + (lane >> 5) * VW);
  }
  const int b_lds = (lane & 31) * LK + (lane >> 5) * VW;

  u4 hreg[H_IT];
  auto load_halo = [&](int chunk) {
    const uint32_t cb = (uint32_t)(chunk * BK * (int)sizeof(T));
    // channel counts that are no multiple of 32: the vectors of the last chunk beyond the row are zeros
    const bool live = chunk * BK + (tid & 3) * VW < g.Cc;
#pragma unroll
    for (int it = 0; it < H_IT; ++it)
      hreg[it] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (live && h_off[it] != kOob) ? h_off[it] + cb : kOob, 0, 0);
  };
  auto store_halo = [&]() {
#pragma unroll
    for (int it = 0; it < H_IT; ++it) {
      const int v = it * kThreads + tid;
      if (v < SLOTS * 4) *(u4 *)&Hs[(v >> 2) * LK + (v & 3) * VW] = hreg[it];
    }
  };
  // weight tile of step t: channels of chunk t / RS at tap t % RS
  int ld_chunk = 0, ld_tap = 0, ld_t = 0;
  const int KT = ((g.Cc + BK - 1) / BK) * RS;
  auto load_b = [&](u4 (&breg)[B_IT]) {
    const uint32_t kb = (uint32_t)((ld_tap * g.Cc + ld_chunk * BK) * (int)sizeof(T));
    const bool live = ld_t < KT && ld_chunk * BK + lkv * VW < g.Cc;  // not into the next tap's weights
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
      if (BN % 64 == 0 || row < BN) *(u4 *)&Bs[buf * (BN * LK) + row * LK + lkv * VW] = breg[i];
    }
  };

  f16v acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

  // Contraction step t = (channel chunk, tap).  A step is two MFMA sub-steps of 16 channels; the
  // fragments of a sub-step are fetched from LDS one sub-step ahead of the MFMAs that use them
  // (sub 1 of step t during sub 0 of step t, sub 0 of step t+1 during sub 1 of step t), so the
  // matrix units do not wait for LDS latency.  The weight tiles form a ring of three in LDS: while
  // step t multiplies, tile t+1 is being read for the next sub-step and tile t+2 is written from
  // registers; one workgroup barrier per step.  Global memory (L2) answers in more cycles than a
  // step lasts, so D weight tiles are in flight in registers: the tile stored to LDS in step t
  // was requested in step t-D.  The patch is single-buffered: at the last tap of a chunk two
  // extra barriers fence its replacement.
  // Tap shift inside the patch: rows advance with r for a forward conv (sr = +1), against it for
  // backward-data (sr = -1); same for columns.
  auto shift_of = [&](int r, int c) {
    const int dh = g.sr > 0 ? r : g.R - 1 - r, dw = g.sr > 0 ? c : g.S - 1 - c;
    return (dh * hg.HC + dw) * LK;
  };
  auto read_sub = [&](int sub, int buf, int shift, u4 (&af)[TM], u4 (&bf)[TN]) {
    const T *bt = Bs + buf * (BN * LK) + b_lds + sub * 2 * VW;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) af[tm] = *(const u4 *)&Hs[a_lds[tm] + shift + sub * 2 * VW];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) bf[tn] = *(const u4 *)&bt[tn * 32 * LK];
  };
  auto mma_sub = [&](const u4 (&af)[TM], const u4 (&bf)[TN]) {
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) mma<T>(bf[tn], af[tm], acc[tm][tn]);
  };

  constexpr int D = TN >= 4 ? 2 : 4;  // weight tiles in flight from global memory (registers permitting)
  u4 rq[D][B_IT];
  u4 fa_a[TM], fa_b[TN];          // fragments of sub-step 0
  u4 fb_a[TM], fb_b[TN];          // fragments of sub-step 1
  int tap_r = 0, tap_s = 0, chunk = 0;  // tap of the step after the current one, chunk in the patch
  int shift_cur = shift_of(0, 0);
  int ring = 0;                   // ring slot of the current step's weight tile
  load_halo(0);
  load_b(rq[0]);
  load_b(rq[1]);
  store_halo();
  load_halo(1);
  store_b(0, rq[0]);
  store_b(1, rq[1]);
#pragma unroll
  for (int i = 0; i < D; ++i) load_b(rq[i]);  // tile 2 + i; step t stores set t % D and refills it with tile t + 2 + D
  __syncthreads();
  read_sub(0, 0, shift_cur, fa_a, fa_b);
  // A wavefront issues in order: LDS reads placed in a burst before the MFMAs leave the matrix unit
  // idle while they issue.  Ask the scheduler to alternate them: one fragment read after each MFMA.
  auto interleave = [&]() {
#pragma unroll
    for (int i = 0; i < TM + TN; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // one LDS read
    }
    __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - TM - TN, 0);
  };
  // one step; `ra` holds tile t+2 (stored to the ring now) and then receives tile t+2+D
  auto step = [&](int t, u4 (&ra)[B_IT]) {
    const int ring1 = ring == 2 ? 0 : ring + 1, ring2 = ring1 == 2 ? 0 : ring1 + 1;
    read_sub(1, ring, shift_cur, fb_a, fb_b);
    if (++tap_s == g.S) {
      tap_s = 0;
      if (++tap_r == g.R) tap_r = 0;
    }
    const bool more = t + 1 < KT;
    const bool swap_patch = more && tap_r == 0 && tap_s == 0;
    shift_cur = shift_of(tap_r, tap_s);
    mma_sub(fa_a, fa_b);
    interleave();
    if (swap_patch) {
      __syncthreads();  // every wavefront has its fragments of the old patch
      ++chunk;
      store_halo();
      load_halo(chunk + 1);
      __syncthreads();
    }
    read_sub(0, ring1, shift_cur, fa_a, fa_b);  // past the last step: a harmless read of live LDS
    mma_sub(fb_a, fb_b);
    interleave();
    store_b(ring2, ra);
    load_b(ra);
    ring = ring1;
    __syncthreads();
  };
  int kt = 0;
  for (; kt + D - 1 < KT; kt += D) {
#pragma unroll
    for (int i = 0; i < D; ++i) step(kt + i, rq[i]);
  }
#pragma unroll
  for (int i = 0; i < D - 1; ++i)
    if (kt + i < KT) step(kt + i, rq[i]);
  // the barrier that ends the last step: patch and weight tiles are dead, their LDS becomes the staging strips
  float *wsums = reinterpret_cast<float *>(smem) + 4 * kStageFloats<TN>;
  store_tile_lds<T, TM, TN, false, STAT>(g, io, rep, m0 + wave * TM * 32, n0, lane, acc,
                                         reinterpret_cast<float *>(smem) + wave * kStageFloats<TN>, wsums + wave * 2 * BN);
  // the workgroup's rows: one partial row per pixel tile
  if (STAT) write_tile_sums<BN, 4>(g, io, rep, hg.tiles, tile, n0, tid, wsums);
}

// Workgroups are handed to the eight XCDs in turn, so ids that differ by 8 share an L2: the column blocks
// of one pixel tile get such ids.  They run at the same time on the same XCD, the patch is fetched into
// that L2 once, and their partial output rows meet there before they are written back.
__device__ __forceinline__ bool halo_block(const HaloGeom &hg, int &tile, int &col) {
  const int per_group = 8 * hg.nb;
  const int group = blockIdx.x / per_group, within = blockIdx.x - group * per_group;
  tile = group * 8 + (within & 7), col = within >> 3;
  return tile < hg.tiles;  // the grid is padded to whole groups
}

// Column blocks 0 .. nb-2 are TN tiles wide, the last one TL <= TN tiles (160 channels = 96 + 64,
// 320 = 128 + 128 + 64): a narrower last block multiplies no padding.
template <int TN, int TL, bool STAT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void k_conv_halo(const ConvGeom g, const GemmIO io,
                                                                                               const HaloGeom hg) {
  __shared__ __attribute__((aligned(16))) char smem[halo_lds_bytes<TN, STAT>()];
  int tile, col;
  if (!halo_block(hg, tile, col)) return;
  if (TL != TN && col == hg.nb - 1)
    conv_halo_body<TL, STAT>(g, io, hg, smem, tile, col);
  else
    conv_halo_body<TN, STAT>(g, io, hg, smem, tile, col);
}
// 64 output channels: few enough registers for three workgroups per compute unit, which hides more of
// the prologue and epilogue of one workgroup behind the matrix work of the others
template <bool STAT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3))) void k_conv_halo_n64(const ConvGeom g,
                                                                                                   const GemmIO io,
                                                                                                   const HaloGeom hg) {
  __shared__ __attribute__((aligned(16))) char smem[halo_lds_bytes<2, STAT>()];
  int tile, col;
  if (!halo_block(hg, tile, col)) return;
  conv_halo_body<2, STAT>(g, io, hg, smem, tile, col);
}

// Stride 2 (forward): 128 output pixels per workgroup, one 32-pixel tile per wavefront.
template <int TN, int TL, bool STAT>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2))) void k_conv_halo_s2(const ConvGeom g, const GemmIO io,
                                                                                                  const HaloGeom hg) {
  __shared__ __attribute__((aligned(16))) char smem[halo_lds_bytes<TN, STAT, kHaloSlotsS2>()];
  int tile, col;
  if (!halo_block(hg, tile, col)) return;
  if (TL != TN && col == hg.nb - 1)
    conv_halo_body<TL, STAT, 1, kHaloSlotsS2, 2>(g, io, hg, smem, tile, col);
  else
    conv_halo_body<TN, STAT, 1, kHaloSlotsS2, 2>(g, io, hg, smem, tile, col);
}

// grid of `tiles` pixel tiles x `nb` column blocks of `bn` channels (the last may be narrower), laid out in
// groups of 8 tiles (see halo_block)
dim3 halo_grid(const ConvGeom &g, int bn, int replicas, HaloGeom &hg) {
  const int bm = g.sp == 2 ? 128 : 256;
  hg.tiles = (g.M + bm - 1) / bm;
  hg.bn = bn;
  hg.nb = (g.N + bn - 1) / bn;
  return dim3((hg.tiles + 7) / 8 * 8 * hg.nb, 1, replicas);
}

template <int TN, int TL>
hipError_t run_halo_s2(hipStream_t st, int replicas, const ConvGeom &g, const GemmIO &io, HaloGeom hg) {
  const dim3 grid = halo_grid(g, TN * 32, replicas, hg);
  if (TN != 3 && io.stat)
    hipLaunchKernelGGL((k_conv_halo_s2<TN, TL, TN != 3>), grid, dim3(kThreads), 0, st, g, io, hg);
  else
    hipLaunchKernelGGL((k_conv_halo_s2<TN, TL, false>), grid, dim3(kThreads), 0, st, g, io, hg);
  return hipGetLastError();
}

template <int TN, int TL>
hipError_t run_halo(hipStream_t st, int replicas, const ConvGeom &g, const GemmIO &io, HaloGeom hg) {
  const dim3 grid = halo_grid(g, TN * 32, replicas, hg);
  if (TN == 4 && io.stat)
    hipLaunchKernelGGL((k_conv_halo<TN, TL, TN == 4>), grid, dim3(kThreads), 0, st, g, io, hg);
  else
    hipLaunchKernelGGL((k_conv_halo<TN, TL, false>), grid, dim3(kThreads), 0, st, g, io, hg);
  return hipGetLastError();
}

bool make_halo_geom(const ConvGeom &g, HaloGeom &hg) {
  const bool s2 = g.sp == 2;
  const int BM = s2 ? 128 : 256;
  if (g.dshift != 0) return false;
  if (s2) {  // forward 3x3, padding 1, even image
    // with few input channels a workgroup is mostly prologue and epilogue, and the kernel that gathers per tap, at
    // three workgroups per compute unit instead of two, is as fast or faster (96 channels: 38 against 44 us)
    static const int min_c = [] {
      const char *e = getenv("PARLE_HALO_S2_MINC");
      return e ? atoi(e) : 128;
    }();
    if (g.Cc < min_c) return false;
    if (g.R != 3 || g.S != 3 || g.off != -1 || g.sr != 1 || 2 * g.P != g.Hin || 2 * g.Q != g.Win) return false;
  } else if (g.sp != 1 || g.P != g.Hin || g.Q != g.Win) {
    return false;
  }
  if (BM % g.Q != 0) return false;
  const int PQ = g.P * g.Q;
  if (PQ >= BM) {
    if (PQ % BM != 0) return false;
    hg.TH = BM / g.Q, hg.nimg = 1;
  } else {
    if (BM % PQ != 0) return false;
    hg.TH = g.P, hg.nimg = BM / PQ;
  }
  hg.HR = g.sp * (hg.TH - 1) + g.R, hg.HC = g.sp * (g.Q - 1) + g.S;
  hg.slots = hg.nimg * hg.HR * hg.HC;
  hg.dImg = make_fastdiv(hg.HR * hg.HC), hg.dHC = make_fastdiv(hg.HC), hg.dRows = make_fastdiv(hg.TH * g.Q);
  const int o_first = g.off, o_last = g.off + (g.R - 1) * g.sr;
  hg.omin_h = o_first < o_last ? o_first : o_last;
  const int w_first = g.off, w_last = g.off + (g.S - 1) * g.sr;
  hg.omin_w = w_first < w_last ? w_first : w_last;
  return hg.slots <= (s2 ? kHaloSlotsS2 : kHaloSlots);
}

}  // namespace

bool conv_halo_applicable(int dtype, const ConvGeom &g, const GemmIO &io, bool out_f32) {
  HaloGeom hg;
  return dtype == 1 && !out_f32 && io.vecA && io.vecB && g.R * g.S > 1 && g.Cc % 8 == 0 && g.Cc >= 16 && g.N % 4 == 0 &&
         io.ldc % 4 == 0 && io.in_bytes > 0 && io.in_bytes < (1LL << 31) && (long long)g.M * io.ldc * 4 < (1LL << 31) && (long long)g.N * g.K * 2 < (1LL << 31) &&
         g.M >= 256 && make_halo_geom(g, hg);
}

namespace {

// Which variant runs a layer.  A launch that wide blocks leave below two workgroups per compute unit runs 64-wide
// ones when those fill the chip in one round at more than two and at most three per unit: every SIMD then holds
// three wavefronts instead of one or two, which overlap each other's LDS reads and MFMAs (128 channels on
// 16 x 16 images, three replicas of 128: -8 %).  With fewer narrow workgroups than that the wide ones are as fast
// or faster.  Otherwise 96- or 128-wide column blocks, whichever pads the output channels least (ties go to the
// wider tile); a last block of at most 64 channels runs two tiles wide.
enum HaloVariant { kHalo64, kHalo96, kHalo128 };
HaloVariant halo_variant(const ConvGeom &g, int replicas) {
  constexpr int kCus = 256;
  const int n = g.N;
  if (g.sp == 2) {  // 128-pixel tiles: one width rule
    if (n <= 64) return kHalo64;
    return (n + 95) / 96 * 96 < (n + 127) / 128 * 128 ? kHalo96 : kHalo128;
  }
  const long long tiles = (g.M + 255) / 256, wide = tiles * ((n + 127) / 128) * replicas,
                  narrow_wgs = tiles * (n / 64) * replicas;
  const bool narrow = n % 64 == 0 && wide < 2 * kCus && narrow_wgs > 2 * kCus && narrow_wgs <= 3 * kCus;
  if (n <= 64 || narrow) return kHalo64;
  const int pad3 = (n + 95) / 96 * 96, pad4 = (n + 127) / 128 * 128;
  return pad3 < pad4 ? kHalo96 : kHalo128;
}

}  // namespace

// Partial rows of column sums (one per pixel tile) a launch with io.stat set writes; 0 where the variant that runs
// the layer does not take them: in the 96-wide epilogue, whose walk visits three channel groups per lane, the
// sums cost more than the reduction pass they replace (160 channels on 32 x 32 images: +0.5 % per step against
// -0.7 % for the other layers of the same network).
int conv_halo_stat_splits(const ConvGeom &g, int replicas) {
  const int bm = g.sp == 2 ? 128 : 256;
  return halo_variant(g, replicas) == kHalo96 ? 0 : (g.M + bm - 1) / bm;
}

hipError_t launch_conv_halo(hipStream_t st, int replicas, const ConvGeom &g, const GemmIO &io) {
  HaloGeom hg;
  if (!make_halo_geom(g, hg)) return hipErrorInvalidValue;
  const int n = g.N;
  if (g.sp == 2) {
    switch (halo_variant(g, replicas)) {
      case kHalo64: return run_halo_s2<2, 2>(st, replicas, g, io, hg);
      case kHalo96: {
        if (io.stat) return hipErrorInvalidValue;
        const int last = n - ((n + 95) / 96 * 96 - 96);
        return last <= 64 ? run_halo_s2<3, 2>(st, replicas, g, io, hg) : run_halo_s2<3, 3>(st, replicas, g, io, hg);
      }
      default: {
        const int last = n - ((n + 127) / 128 * 128 - 128);
        return last <= 64 ? run_halo_s2<4, 2>(st, replicas, g, io, hg) : run_halo_s2<4, 4>(st, replicas, g, io, hg);
      }
    }
  }
  switch (halo_variant(g, replicas)) {
    case kHalo64: {
      const dim3 grid = halo_grid(g, 64, replicas, hg);
      if (io.stat)
        hipLaunchKernelGGL(k_conv_halo_n64<true>, grid, dim3(kThreads), 0, st, g, io, hg);
      else
        hipLaunchKernelGGL(k_conv_halo_n64<false>, grid, dim3(kThreads), 0, st, g, io, hg);
      return hipGetLastError();
    }
    case kHalo96: {
      if (io.stat) return hipErrorInvalidValue;  // see conv_halo_stat_splits
      const int last = n - ((n + 95) / 96 * 96 - 96);
      return last <= 64 ? run_halo<3, 2>(st, replicas, g, io, hg) : run_halo<3, 3>(st, replicas, g, io, hg);
    }
    default: {
      const int last = n - ((n + 127) / 128 * 128 - 128);
      return last <= 64 ? run_halo<4, 2>(st, replicas, g, io, hg) : run_halo<4, 4>(st, replicas, g, io, hg);
    }
  }
}
