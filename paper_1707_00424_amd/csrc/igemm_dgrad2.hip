// Backward-data of a stride-2 3x3 convolution with padding 1 (bf16), all four parity classes of a block of
// input pixels in one workgroup.
//
// An input pixel (h, w) of such a layer is reached by the taps whose parity matches its own: one tap for
// (even, even), two for (even, odd) and (odd, even), four for (odd, odd) -- 9/4 of a tap per pixel on
// average, a short contraction.  The pass is bound by its memory traffic (the ReLU mask read and the
// gradient written, one pixel row each per output row), so what matters is that this traffic is contiguous:
// a kernel that gives every workgroup pixels of ONE class (so that its rows share their taps) reads and
// writes every other pixel, half of every cache line at a time.  Here a workgroup owns a block of 16 x 16
// input pixels = 8 x 8 positions (i, j) of the output-gradient grid x 4 classes, one class per wavefront:
//   dx[2i + a, 2j + c] = sum over the taps (r, s) of class (a, c) of dy[i + di(r), j + dj(s)] . w[:, r, s, :]
//   a = 0: r = 1, di = 0;   a = 1: r = 0, di = 1 and r = 2, di = 0   (columns alike)
// The four wavefronts write the interleaved pixels of the same rows at the same time, so whole lines form in
// L2, and they share one staged patch of dy for all their shifted taps.
#include <stdlib.h>

#include "igemm_dev.h"

namespace {

using namespace igemm_dev;

constexpr uint32_t kOob = 0x80000000u;

// Per 32-channel chunk of the contraction the workgroup stages, with coalesced 16-byte loads, the 9 x 9 patch
// of dy positions that its block and the shifted taps touch and the weight tiles of all nine taps; every
// wavefront then multiplies the taps of its own class from LDS.  The next chunk travels from memory to
// registers meanwhile; LDS is single-buffered (two barriers per chunk).
constexpr int kLK = 40;          // LDS row pitch in elements: 32 channels + 8 of padding (80 bytes)
constexpr int kPatchSlots = 81;  // (8 + 1) x (8 + 1) positions

template <int TN>
constexpr int dgrad_lds_bytes() {
  constexpr int pipe = (kPatchSlots + 9 * TN * 32) * kLK * 2;
  constexpr int stage = 4 * kStageFloats<TN> * (int)sizeof(float);
  return pipe > stage ? pipe : stage;
}

template <int TN>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(3))) void k_dgrad_s2(const ConvGeom g, const GemmIO io, const int rot_mask) {
  typedef bf16_t T;
  constexpr int TM = 2, BN = TN * 32;
  constexpr int H_IT = (kPatchSlots * 4 + kThreads - 1) / kThreads;  // 16-byte vectors per thread: patch
  constexpr int B_IT = (9 * BN * 4 + kThreads - 1) / kThreads;       // and weight tiles
  __shared__ __attribute__((aligned(16))) char smem[dgrad_lds_bytes<TN>()];
  T *Hs = reinterpret_cast<T *>(smem);                       // patch: slot (ti, tj) at (ti*9 + tj) * kLK
  T *Bs = Hs + kPatchSlots * kLK;                            // tap t, row n at (t*BN + n) * kLK

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rep = blockIdx.z, tile = blockIdx.x, n0 = blockIdx.y * BN;
  // Parity class of this wavefront's pixels.  Wavefront i of every workgroup lands on SIMD i, and the classes differ
  // in work (1, 2, 2, 4 taps): the assignment rotates with the tile so that no SIMD collects the four-tap class of
  // every workgroup on its compute unit.
  // (workgroup ids 8 apart share an XCD: the rotation is taken from the id within the XCD, mixed so that neither
  // a round-robin over the 32 compute units nor a blocked assignment lines the classes up again)
  const int kx = tile >> 3;
  const int cls = (wave + ((kx + (kx >> 2) + (kx >> 5)) & rot_mask)) & 3;
  const int a = cls >> 1, c = cls & 1;
  const int row_l = lane & 31, h = lane >> 5;
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.in + rep * io.in_rs), 0, (int)(io.in_bytes), 0x00020000);
  const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.w + rep * io.w_rs), 0, (int)((long long)g.N * g.K * sizeof(T)), 0x00020000);

  // block of the tile: image b, block row bi, block column bj (blocks of 8 x 8 positions)
  const int lbw = g.plq - 4, lblk = g.plp - 4 + lbw;
  const int b = tile >> lblk, blk = tile & ((1 << lblk) - 1);
  const int bi = blk >> lbw, bj = blk & ((1 << lbw) - 1);

  // loader: vector v = it*256 + tid; patch slot v/4 (channels 8*(v%4) .. +7 of the chunk), weight row v/4
  uint32_t h_off[H_IT], w_off[B_IT];
#pragma unroll
  for (int it = 0; it < H_IT; ++it) {
    const int v = it * kThreads + tid, slot = v >> 2;
    const int i = bi * 8 + slot / 9, j = bj * 8 + slot % 9;
    h_off[it] = (slot < kPatchSlots && i < g.Hin && j < g.Win)
                    ? (uint32_t)((((b * g.Hin + i) * g.Win + j) * g.Cc + (v & 3) * 8) * (int)sizeof(T))
                    : kOob;
  }
#pragma unroll
  for (int it = 0; it < B_IT; ++it) {
    const int v = it * kThreads + tid, row = v >> 2;
    const int t = row / BN, n = n0 + row - t * BN;
    w_off[it] = (row < 9 * BN && n < g.N) ? (uint32_t)((n * g.K + t * g.Cc + (v & 3) * 8) * (int)sizeof(T)) : kOob;
  }
  auto load_chunk = [&](int ch, u4 (&hq)[H_IT], u4 (&wq)[B_IT]) {
    const uint32_t cb = (uint32_t)(ch * 32 * (int)sizeof(T));
#pragma unroll
    for (int it = 0; it < H_IT; ++it)
      hq[it] = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, h_off[it] == kOob ? kOob : h_off[it] + cb, 0, 0);
#pragma unroll
    for (int it = 0; it < B_IT; ++it)
      wq[it] = __builtin_amdgcn_raw_buffer_load_b128(b_rsrc, w_off[it] == kOob ? kOob : w_off[it] + cb, 0, 0);
  };
  auto store_chunk = [&](const u4 (&hq)[H_IT], const u4 (&wq)[B_IT]) {
#pragma unroll
    for (int it = 0; it < H_IT; ++it) {
      const int v = it * kThreads + tid;
      if (v < kPatchSlots * 4) *(u4 *)&Hs[(v >> 2) * kLK + (v & 3) * 8] = hq[it];
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int v = it * kThreads + tid;
      if ((9 * BN * 4) % kThreads == 0 || v < 9 * BN * 4) *(u4 *)&Bs[(v >> 2) * kLK + (v & 3) * 8] = wq[it];
    }
  };

  // fragment rows of this lane: position tm*32 + row_l of the block -> patch slot of shift (0, 0)
  int a_slot[TM];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    const int pos = tm * 32 + row_l;
    a_slot[tm] = ((pos >> 3) * 9 + (pos & 7)) * kLK + 8 * h;
  }
  const int b_row = row_l * kLK + 8 * h;
  // taps of the class: nr x ns of them; tap t -> window row r, dy row shift di (columns alike)
  const int nr = a ? 2 : 1, ns = c ? 2 : 1, ntaps = nr * ns;

  f16v acc[TM][TN];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

  const int chunks = g.Cc >> 5;
  u4 hq[H_IT], wq[B_IT];
  load_chunk(0, hq, wq);
  store_chunk(hq, wq);
  __syncthreads();
  for (int ch = 0; ch < chunks; ++ch) {
    if (ch + 1 < chunks) load_chunk(ch + 1, hq, wq);
    for (int t = 0; t < ntaps; ++t) {  // wavefront-uniform
      const int tr = t / ns, ts = t - tr * ns;
      const int r = a ? 2 * tr : 1, di = a ? 1 - tr : 0;
      const int sc = c ? 2 * ts : 1, dj = c ? 1 - ts : 0;
      const T *ap = Hs + (di * 9 + dj) * kLK;
      const T *bp = Bs + (r * 3 + sc) * BN * kLK + b_row;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        u4 af[TM], bf[TN];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) af[tm] = *(const u4 *)&ap[a_slot[tm] + sub * 16];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) bf[tn] = *(const u4 *)&bp[tn * 32 * kLK + sub * 16];
        // operands swapped: every accumulator holds the transposed tile (four consecutive channels of a pixel
        // per lane), the layout the epilogue expects
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
          for (int tn = 0; tn < TN; ++tn) mma<T>(bf[tn], af[tm], acc[tm][tn]);
      }
    }
    __syncthreads();  // every wavefront has read the chunk (after the last one: LDS becomes the staging strips)
    if (ch + 1 < chunks) {
      store_chunk(hq, wq);
      __syncthreads();
    }
  }

  store_tile_lds<T, TM, TN, false>(g, io, rep, tile * 256 + cls * 64, n0, lane, acc,
                                   reinterpret_cast<float *>(smem) + wave * kStageFloats<TN>);
}

int exact_log2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return (1 << l) == v ? l : -1;
}

template <int TN>
hipError_t run_dgrad_s2(hipStream_t st, int replicas, const ConvGeom &g, const GemmIO &io) {
  dim3 grid(g.M / 256, (g.N + TN * 32 - 1) / (TN * 32), replicas);
  static const int rot = [] {
    const char *e = getenv("PARLE_S2_ROT");
    return e ? atoi(e) : 3;
  }();
  hipLaunchKernelGGL((k_dgrad_s2<TN>), grid, dim3(kThreads), 0, st, g, io, rot);
  return hipGetLastError();
}

}  // namespace

// g: backward-data geometry (conv_bwd_geom) of a stride-2 layer.
bool dgrad_s2_applicable(int dtype, const ConvGeom &g, const GemmIO &io, bool out_f32) {
  return dtype == 1 && !out_f32 && g.dshift == 1 && g.R == 3 && g.S == 3 && g.off == 1 && g.sr == -1 && g.sp == 1 &&
         exact_log2(g.P) >= 4 && exact_log2(g.Q) >= 4 && g.P == 2 * g.Hin && g.Q == 2 * g.Win && g.Cc % 32 == 0 &&
         g.N % 4 == 0 && io.ldc % 4 == 0 && io.vecA && io.vecB && io.in_bytes > 0 && io.in_bytes < (1LL << 31) &&
         (long long)g.M * io.ldc * 4 < (1LL << 31) && (long long)g.N * g.K * 2 < (1LL << 31) && g.M % 256 == 0;
}

hipError_t launch_dgrad_s2(hipStream_t st, int replicas, const ConvGeom &g_in, const GemmIO &io) {
  ConvGeom g = g_in;
  g.plp = exact_log2(g.P), g.plq = exact_log2(g.Q), g.pblk = 1;  // rows ordered block, class, position
  // 64-wide column blocks: three workgroups fit a compute unit (registers and LDS), which measured faster than
  // 96-wide blocks at two per unit also for 96 and 192 channels
  return run_dgrad_s2<2>(st, replicas, g, io);
}
