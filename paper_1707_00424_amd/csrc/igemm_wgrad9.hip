// Backward-weight of stride-1 "same" 3x3 convolutions (bf16) with the input patch staged ONCE in LDS
// and each output-gradient fragment reused by all nine window taps.
//
//   dW[n][r][s][c] = sum over pixels (b, p, q) of dy[b, p, q, n] * x[b, p + r - 1, q + s - 1, c]
//
// The contraction runs over pixels, which is the slow index of both operands in memory
// ([pixel][channel]); MFMA fragments need it contiguous, so they are fetched with the LDS transpose
// read (ds_read_b64_tr_b16), which delivers about half the bandwidth of a plain 16-byte read.  The
// kernel is built to need few of them:
//   * a wavefront owns one 32-channel tile of dy, one 32-channel tile of x and ALL nine taps
//     (nine 32x32 accumulators): one dy fragment serves nine MFMAs;
//   * a contraction sub-step is one row of 16 pixels; the x fragment of (row j, column shift s) is
//     the operand of tap (r, s) for dy row j + 1 - r, so the fragments of three consecutive x rows are
//     kept in registers and each dy row reads only the three fragments of the row that enters;
//   * per 9 MFMAs: 1 + 3 fragment reads (0.44 KiB of LDS traffic per MFMA instead of 1 KiB for a
//     plain 64x64 wavefront tile), and the patch is fetched from memory once, not once per tap.
// Images 8 pixels wide take sub-steps of two rows of 8 pixels: the fragment of the row pair that
// starts at x row t serves tap row r of the dy pair that starts at row t + 1 - r, pairs start at
// even dy rows, so one of three fragment sets is reused and two enter per sub-step.
// A workgroup is NT wavefronts (NT dy tiles sharing one x tile).  It walks blocks of 128 pixels
// (8 rows x 16 columns, or two 8 x 8 images) of the images of its split; the operands of the next block travel from memory to
// registers while the current block is multiplied, LDS is single-buffered.  Partial sums of the
// splits go to per-split buffers that a second kernel adds in a fixed order (no float atomics).
// BIAS: the workgroups of the first x tile also sum the dy vectors they stage (a thread keeps the same eight
// channels for the whole kernel) and write the layer's bias gradient, the column sums of dy, behind the weights.
#include "igemm_dev.h"

namespace {

using namespace igemm_dev;
typedef short s4v __attribute__((ext_vector_type(4)));

constexpr int kBlockPixels = 128;                // 8 rows x 16 columns, or two images of 8 x 8
constexpr int kSub = 8;                          // contraction sub-steps (16 pixels) per block
constexpr int kXS = 96;                          // bytes per patch pixel: 32 channels + padding
// patch of a block: one halo pixel around each image part
template <int KC>
struct Patch {
  static constexpr int PC = KC + 2;                      // columns
  static constexpr int IMG = KC == 16 ? 1 : 2;           // image parts per block
  static constexpr int PRI = kBlockPixels / KC / IMG + 2;  // rows per image part
  static constexpr int SLOTS = IMG * PRI * PC;           // 180 / 200
};

struct Wg9Geom {
  int H, W, Cin, N;          // image, channels in / out
  int B;                     // images per replica
  int bpi, cbn;              // blocks per image, column blocks per image row
  int total_blocks, bps;     // per replica; blocks per split
  int splits;
  FastDiv dBpi, dCbn;
};

__device__ __forceinline__ u4 tr_frag(const bf16_t *tile, int ld, int krow, int col) {
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

template <int NT, int KC, bool BIAS>
__global__ __launch_bounds__(NT * 64) __attribute__((amdgpu_waves_per_eu(2))) void k_wgrad9(const Wg9Geom wg, const WgradIO io) {
  typedef Patch<KC> PT;
  constexpr int kSlots = PT::SLOTS, kPC = PT::PC;
  constexpr int T = NT * 64;
  constexpr int DS = NT * 64 + 32;                        // bytes per dy pixel row in LDS
  constexpr int X_IT = (kSlots * 4 + T - 1) / T;          // 16-byte vectors of the patch per thread
  constexpr int D_IT = kSub;                              // dy: 16 pixels per iteration
  __shared__ __attribute__((aligned(16))) char xs[kSlots * kXS];
  __shared__ __attribute__((aligned(16))) char ds[kBlockPixels * DS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ct = blockIdx.x, ng = blockIdx.y;
  const int rep = blockIdx.z / wg.splits, split = blockIdx.z - rep * wg.splits;
  const int blk_begin = split * wg.bps, blk_end = min(wg.total_blocks, blk_begin + wg.bps);
  const long long x_bytes = (long long)wg.B * wg.H * wg.W * wg.Cin * 2, dy_bytes = (long long)wg.B * wg.H * wg.W * wg.N * 2;
  const __amdgpu_buffer_rsrc_t x_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)((const bf16_t *)io.x + rep * io.x_rs), 0, (int)x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t d_rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)((const bf16_t *)io.dy + rep * io.dy_rs), 0, (int)dy_bytes, 0x00020000);

  // patch loader: vector id = it*T + tid covers patch slot id/4 = (image part, row, column), channels 8*(id%4) .. +7
  int x_rel[X_IT], x_prow[X_IT], x_pcol[X_IT], x_img[X_IT];
#pragma unroll
  for (int it = 0; it < X_IT; ++it) {
    const int id = it * T + tid, slot = id >> 2;
    const int img = slot / (PT::PRI * kPC), rem = slot - img * (PT::PRI * kPC);
    const int prow = rem / kPC, pcol = rem - prow * kPC;
    x_prow[it] = slot < kSlots ? prow : -1000;   // never a valid image row
    x_pcol[it] = pcol;
    x_img[it] = img;
    x_rel[it] = (((img * wg.H + prow - 1) * wg.W + (pcol - 1)) * wg.Cin + (id & 3) * 8) * 2;
  }
  // dy loader: iteration `it` covers 16 pixels of the block (one row of 16, or two rows of 8, which
  // are consecutive in memory); this thread's pixel inside them and its channel vector are fixed
  const int d_vec = tid % (NT * 4), d_pcol = tid / (NT * 4);
  const int d_rel = (d_pcol * wg.N + (ng * NT * 32 + d_vec * 8)) * 2;
  const int d_pitch = (KC == 16 ? wg.W : 16) * wg.N * 2;

  u4 xreg[X_IT], dreg[D_IT];
  const bool tally = BIAS && ct == 0;
  float bsum[BIAS ? 8 : 1];
  if (BIAS) {
#pragma unroll
    for (int e = 0; e < 8; ++e) bsum[e] = 0.f;
  }
  auto load_block = [&](int blk) {
    const bool live = blk < blk_end;
    int b, row0, col0;
    if (KC == 16) {
      b = (int)fdiv((uint32_t)(live ? blk : 0), wg.dBpi);
      const int rem = (live ? blk : 0) - b * wg.bpi;
      const int rb = (int)fdiv((uint32_t)rem, wg.dCbn), cb = rem - rb * wg.cbn;
      row0 = rb * 8, col0 = cb * 16;
    } else {
      b = 2 * (live ? blk : 0), row0 = 0, col0 = 0;
    }
    const int xbase = (((b * wg.H + row0) * wg.W + col0) * wg.Cin + ct * 32) * 2;
#pragma unroll
    for (int it = 0; it < X_IT; ++it) {
      const int row = row0 + x_prow[it] - 1, col = col0 + x_pcol[it] - 1;
      const bool ok = live && (unsigned)row < (unsigned)wg.H && (unsigned)col < (unsigned)wg.W && b + x_img[it] < wg.B;
      xreg[it] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, ok ? (uint32_t)(xbase + x_rel[it]) : kOobOffset, 0, 0);
    }
    // an image beyond the batch (odd batch, second 8 x 8 image of the last block) lies beyond the buffer: zeros
    const int dbase = ((b * wg.H + row0) * wg.W + col0) * wg.N * 2;
#pragma unroll
    for (int it = 0; it < D_IT; ++it)
      dreg[it] = __builtin_amdgcn_raw_buffer_load_b128(d_rsrc, live ? (uint32_t)(dbase + it * d_pitch + d_rel) : kOobOffset, 0, 0);
  };
  auto store_block = [&]() {
#pragma unroll
    for (int it = 0; it < X_IT; ++it) {
      const int id = it * T + tid;
      if (kSlots * 4 % T == 0 || id < kSlots * 4) *(u4 *)&xs[(id >> 2) * kXS + (id & 3) * 16] = xreg[it];
    }
#pragma unroll
    for (int it = 0; it < D_IT; ++it) *(u4 *)&ds[(it * 16 + d_pcol) * DS + d_vec * 16] = dreg[it];
    if (BIAS && tally) {
#pragma unroll
      for (int it = 0; it < D_IT; ++it) {
        const uint32_t w[4] = {dreg[it].x, dreg[it].y, dreg[it].z, dreg[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          bsum[2 * e] += __uint_as_float(w[e] << 16);
          bsum[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
        }
      }
    }
  };

  f16v acc[3][3];
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int c = 0; c < 3; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

  // fragment addressing of the transpose read: 16-lane group gq covers columns 16*(gq%2) .. +15 and
  // contraction half gq/2
  const int gq = lane >> 4, j = lane & 15;
  const int frag_k = 8 * (gq >> 1) + (j >> 2), frag_c = 16 * (gq & 1) + 4 * (j & 3);
  // contraction index e of the sub-step -> patch slot: one row of 16, or two rows of 8 (e / 8 is the
  // lane's contraction half gq / 2; the transpose read adds 4 slots for its second part)
  const int frag_x = KC == 16 ? frag_k : (gq >> 1) * kPC + (j >> 2);
  const bf16_t *xt = (const bf16_t *)xs, *dt = (const bf16_t *)ds + wave * 32;
  // x fragments of the sub-step whose first pixel is patch row `prow`, at the three column shifts;
  // dy fragment of sub-step p
  auto read_x = [&](int prow, u4 (&f)[3]) {
#pragma unroll
    for (int s = 0; s < 3; ++s) f[s] = tr_frag(xt + (prow * kPC + s) * (kXS / 2), kXS / 2, frag_x, frag_c);
  };
  auto read_d = [&](int p) { return tr_frag(dt + p * 16 * (DS / 2), DS / 2, frag_k, frag_c); };

  load_block(blk_begin);
  for (int blk = blk_begin; blk < blk_end; ++blk) {
    __syncthreads();  // every wavefront has read the fragments of the previous block
    store_block();
    __syncthreads();
    load_block(blk + 1);
    u4 window[3][3], dfrag[2];
    if (KC == 16) {
      // x rows p-1, p, p+1 live in window[(p + 0, 1, 2) % 3]; patch row index = image row + 1
      read_x(0, window[0]);
      read_x(1, window[1]);
      read_x(2, window[2]);
      dfrag[0] = read_d(0);
#pragma unroll
      for (int p = 0; p < kSub; ++p) {
        const int w0 = p % 3, w1 = (p + 1) % 3, w2 = (p + 2) % 3;
        const u4 d = dfrag[p & 1];
        // taps of window row r = 0 use x row p-1; its registers then take x row p+2 for the next rows
#pragma unroll
        for (int s = 0; s < 3; ++s) mma<bf16_t>(d, window[w0][s], acc[0][s]);
        if (p + 1 < kSub) dfrag[(p + 1) & 1] = read_d(p + 1);
        u4 incoming[3];
        if (p + 2 < kSub + 1) read_x(p + 3, incoming);
#pragma unroll
        for (int s = 0; s < 3; ++s) mma<bf16_t>(d, window[w1][s], acc[1][s]);
#pragma unroll
        for (int s = 0; s < 3; ++s) mma<bf16_t>(d, window[w2][s], acc[2][s]);
        if (p + 2 < kSub + 1) {
#pragma unroll
          for (int s = 0; s < 3; ++s) window[w0][s] = incoming[s];
        }
      }
    } else {
      // the dy pair that starts at image row 2*mu meets the x pairs that start at patch rows 2*mu + r
      // (patch row = image row + 1); pair t lives in window[t % 3]
#pragma unroll
      for (int img = 0; img < 2; ++img) {
        const int pr0 = img * PT::PRI;
        read_x(pr0 + 0, window[0]);
        read_x(pr0 + 1, window[1]);
        read_x(pr0 + 2, window[2]);
        dfrag[0] = read_d(img * 4);
#pragma unroll
        for (int mu = 0; mu < 4; ++mu) {
          const int w0 = (2 * mu) % 3, w1 = (2 * mu + 1) % 3, w2 = (2 * mu + 2) % 3;
          const u4 d = dfrag[mu & 1];
#pragma unroll
          for (int s = 0; s < 3; ++s) mma<bf16_t>(d, window[w0][s], acc[0][s]);
          if (mu + 1 < 4) dfrag[(mu + 1) & 1] = read_d(img * 4 + mu + 1);
          u4 in0[3], in1[3];
          if (mu + 1 < 4) read_x(pr0 + 2 * mu + 3, in0);
#pragma unroll
          for (int s = 0; s < 3; ++s) mma<bf16_t>(d, window[w1][s], acc[1][s]);
          if (mu + 1 < 4) read_x(pr0 + 2 * mu + 4, in1);
#pragma unroll
          for (int s = 0; s < 3; ++s) mma<bf16_t>(d, window[w2][s], acc[2][s]);
          if (mu + 1 < 4) {
#pragma unroll
            for (int s = 0; s < 3; ++s) window[w0][s] = in0[s], window[w1][s] = in1[s];
          }
        }
      }
    }
  }

  // acc[r][s]: lane holds column c = lane % 32 and rows n = 8*(v/4) + 4*(lane/32) + v%4
  float *out = io.out + rep * io.out_rs + split * io.split_stride;
  const int c = ct * 32 + (lane & 31), h = lane >> 5;
  const int K = 9 * wg.Cin;
#pragma unroll
  for (int r = 0; r < 3; ++r)
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int n = (ng * NT + wave) * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
        out[(long long)n * K + (r * 3 + s) * wg.Cin + c] = acc[r][s][v];
      }
  if (BIAS && tally) {
    // the sixteen threads that share a channel vector (one per pixel column of a sub-step) are added in a fixed order
    float *bs = (float *)ds;  // [16][NT * 32]
    __syncthreads();          // the last block's fragments have been read
#pragma unroll
    for (int e = 0; e < 8; ++e) bs[d_pcol * (NT * 32) + d_vec * 8 + e] = bsum[e];
    __syncthreads();
    if (tid < NT * 32) {
      float t = 0.f;
#pragma unroll
      for (int q = 0; q < 16; ++q) t += bs[q * (NT * 32) + tid];
      out[(long long)wg.N * K + ng * NT * 32 + tid] = t;
    }
  }
}

int wg9_tiles(int nt32) {  // dy tiles per workgroup for N/32 tiles in all
  // four first: two workgroups of four wavefronts fill a compute unit's eight wavefront slots (two per SIMD at
  // this kernel's register count), one of five leaves three of them empty
  static const int order[4] = {4, 5, 3, 2};
  for (int nt : order)
    if (nt32 % nt == 0) return nt;
  return nt32 == 1 ? 1 : 0;
}

bool make_wg9_geom(const ConvGeom &g, int batch_hint, Wg9Geom &wg) {
  (void)batch_hint;
  wg.H = g.Hin, wg.W = g.Win, wg.Cin = g.Cc, wg.N = g.N;
  wg.B = g.M / (g.P * g.Q);
  if (wg.W == 8) {  // two whole images per block
    wg.cbn = 1, wg.bpi = 1;
    wg.total_blocks = (wg.B + 1) / 2;
  } else {
    wg.cbn = wg.W / 16;
    wg.bpi = (wg.H / 8) * wg.cbn;
    wg.total_blocks = wg.B * wg.bpi;
  }
  wg.dBpi = make_fastdiv(wg.bpi), wg.dCbn = make_fastdiv(wg.cbn);
  return true;
}

}  // namespace

bool wgrad9_applicable(int dtype, const ConvGeom &g) {
  if (dtype != 1 || g.R != 3 || g.S != 3 || g.sp != 1 || g.dshift != 0 || g.sr != 1 || g.off != -1) return false;
  if (g.P != g.Hin || g.Q != g.Win) return false;
  if (!((g.Win % 16 == 0 && g.Hin % 8 == 0) || (g.Win == 8 && g.Hin == 8))) return false;
  if (g.Cc % 32 != 0 || g.N % 32 != 0 || wg9_tiles(g.N / 32) < 2) return false;
  const long long in_bytes = (long long)g.M * g.Cc * 2, dy_bytes = (long long)g.M * g.N * 2;
  return in_bytes < (1LL << 31) && dy_bytes < (1LL << 31) && g.M % (g.P * g.Q) == 0;
}

// Blocks of 128 pixels per split so that the launch fills the chip; returns the split count and the
// pixels per split in *chunk_out.
int wgrad9_plan(int replicas, const ConvGeom &g, int *chunk_out) {
  Wg9Geom wg;
  make_wg9_geom(g, 0, wg);
  const int nt = wg9_tiles(g.N / 32);
  const long long tiles = (long long)(g.Cc / 32) * (g.N / 32 / nt) * replicas;
  // about 1024 wavefronts in flight (one per SIMD; more splits cost more in partial sums than they gain), never
  // fewer than 4 blocks per split
  static const int waves = [] {
    const char *e = getenv("PARLE_WG9_WAVES");
    const int v = e ? atoi(e) : 0;
    return v > 0 ? v : 1024;
  }();
  const int target = g.leaf_waves > 0 ? g.leaf_waves : waves;
  long long want = (target / nt + tiles - 1) / tiles;
  if (want > wg.total_blocks / 4) want = wg.total_blocks / 4;
  if (want < 1) want = 1;
  const long long cap = 65535 / replicas;
  if (want > cap) want = cap;
  const int bps = (int)((wg.total_blocks + want - 1) / want);
  const int splits = (wg.total_blocks + bps - 1) / bps;
  if (chunk_out) *chunk_out = bps * kBlockPixels;
  return splits;
}

hipError_t launch_wgrad9(hipStream_t st, int replicas, const ConvGeom &g, const WgradIO &io) {
  Wg9Geom wg;
  make_wg9_geom(g, 0, wg);
  wg.bps = io.chunk / kBlockPixels;
  wg.splits = io.splits;
  if (wg.bps < 1 || (long long)wg.bps * io.splits < wg.total_blocks) return hipErrorInvalidValue;
  const int nt = wg9_tiles(g.N / 32);
  dim3 grid(g.Cc / 32, g.N / 32 / nt, replicas * io.splits);
#define WG9_LAUNCH(NTV, KCV)                                                                  \
  do {                                                                                        \
    if (io.with_bias)                                                                         \
      hipLaunchKernelGGL((k_wgrad9<NTV, KCV, true>), grid, dim3(NTV * 64), 0, st, wg, io);    \
    else                                                                                      \
      hipLaunchKernelGGL((k_wgrad9<NTV, KCV, false>), grid, dim3(NTV * 64), 0, st, wg, io);   \
  } while (0)
#define WG9_CASE(NTV)          \
  case NTV:                    \
    if (wg.W == 8)             \
      WG9_LAUNCH(NTV, 8);      \
    else                       \
      WG9_LAUNCH(NTV, 16);     \
    break
  switch (nt) {
    WG9_CASE(2);
    WG9_CASE(3);
    WG9_CASE(4);
    WG9_CASE(5);
    default: return hipErrorInvalidValue;
  }
#undef WG9_CASE
#undef WG9_LAUNCH
  return hipGetLastError();
}
