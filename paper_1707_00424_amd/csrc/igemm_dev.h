// Device-side helpers shared by the implicit-GEMM kernels (MFMA wrappers, LDS fragment reads).
#pragma once
#include "igemm.h"

namespace igemm_dev {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv &f) {
  return (uint32_t)(((uint64_t)n * f.magic) >> f.shift);
}

template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) {
  return v;
}
template <>
__device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) {
  return bf16_to_f32(v);
}
template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) {
  return v;
}
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) {
  return f32_to_bf16(v);
}

// One contraction sub-step on a 32x32 accumulator from two 16-byte fragments.
template <typename T>
__device__ __forceinline__ void mma(const u4 &a, const u4 &b, f16v &acc);
template <>
__device__ __forceinline__ void mma<float>(const u4 &a, const u4 &b, f16v &acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma<bf16_t>(const u4 &a, const u4 &b, f16v &acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), acc, 0, 0, 0);
}

template <typename T, int VW>
__device__ __forceinline__ u4 pack_vec(const T *tmp) {
  u4 r;
  if (sizeof(T) == 4) {
    const uint32_t *p = (const uint32_t *)tmp;
    r.x = p[0], r.y = p[1], r.z = p[2], r.w = p[3];
  } else {
    const unsigned short *p = (const unsigned short *)tmp;
    r.x = p[0] | ((uint32_t)p[1] << 16);
    r.y = p[2] | ((uint32_t)p[3] << 16);
    r.z = p[4] | ((uint32_t)p[5] << 16);
    r.w = p[6] | ((uint32_t)p[7] << 16);
  }
  return r;
}

__device__ __forceinline__ bool tap(int t, int dshift, int lim, int &idx) {
  const int dm = (1 << dshift) - 1;
  idx = t >> dshift;
  return t >= 0 && (t & dm) == 0 && idx < lim;
}

// Row index of a tile -> pixel index (b*P + p)*Q + q, for geometries with parity-class row order.
__device__ __forceinline__ uint32_t row_pixel(const ConvGeom &g, uint32_t m) {
  if (g.plq == 0) return m;
  const int lpq = g.plp + g.plq;
  const uint32_t b = m >> lpq, mi = m & ((1u << lpq) - 1u);
  if (g.pblk) {
    const uint32_t blk = mi >> 8, cls = (mi >> 6) & 3u, i = (mi >> 3) & 7u, j = mi & 7u;
    const uint32_t bi = blk >> (g.plq - 4), bj = blk & ((1u << (g.plq - 4)) - 1u);
    return (b << lpq) | ((16u * bi + 2u * i + (cls >> 1)) << g.plq) | (16u * bj + 2u * j + (cls & 1u));
  }
  const uint32_t cls = mi >> (lpq - 2), rem = mi & ((1u << (lpq - 2)) - 1u);
  const uint32_t ph = rem >> (g.plq - 1), qh = rem & ((1u << (g.plq - 1)) - 1u);
  return (b << lpq) | ((2u * ph + (cls >> 1)) << g.plq) | (2u * qh + (cls & 1u));
}

// Shared MFMA inner step: every wavefront multiplies its TM x TN fragments for both halves of BK.
template <typename T, int TM, int TN, int LK, int VW>
__device__ __forceinline__ void mma_tile(const T *As, const T *Bs, int arow0, int brow0, int lane, f16v (&acc)[TM][TN]) {
  const int r = lane & 31, h = lane >> 5;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    u4 af[TM], bf[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) af[tm] = *(const u4 *)&As[(arow0 + tm * 32 + r) * LK + sub * 2 * VW + h * VW];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) bf[tn] = *(const u4 *)&Bs[(brow0 + tn * 32 + r) * LK + sub * 2 * VW + h * VW];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) mma<T>(af[tm], bf[tn], acc[tm][tn]);
  }
}


// Same inner step with the MFMA operands swapped: every 32x32 accumulator then holds the TRANSPOSED
// tile (lane l: row m = l % 32; registers v: columns 8*(v/4) + 4*(l/32) + v%4), i.e. each lane owns
// groups of four consecutive output channels of one pixel and can store them as one vector.
template <typename T, int TM, int TN, int LK, int VW>
__device__ __forceinline__ void mma_tile_t(const T *As, const T *Bs, int arow0, int brow0, int lane, f16v (&acc)[TM][TN]) {
  const int r = lane & 31, h = lane >> 5;
#pragma unroll
  for (int sub = 0; sub < 2; ++sub) {
    u4 af[TM], bf[TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) af[tm] = *(const u4 *)&As[(arow0 + tm * 32 + r) * LK + sub * 2 * VW + h * VW];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) bf[tn] = *(const u4 *)&Bs[(brow0 + tn * 32 + r) * LK + sub * 2 * VW + h * VW];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) mma<T>(bf[tn], af[tm], acc[tm][tn]);
  }
}

template <typename T>
struct Vec4;  // four consecutive elements of an activation tensor
template <>
struct Vec4<float> {
  typedef f4 type;
  static __device__ __forceinline__ f4 to_f32(f4 v) { return v; }
  static __device__ __forceinline__ f4 from_f32(f4 v) { return v; }
};
template <>
struct Vec4<bf16_t> {
  typedef us4 type;
  static __device__ __forceinline__ f4 to_f32(us4 v) {
    f4 r = {bf16_to_f32(v.x), bf16_to_f32(v.y), bf16_to_f32(v.z), bf16_to_f32(v.w)};
    return r;
  }
  static __device__ __forceinline__ us4 from_f32(f4 v) {
    return f32x4_to_bf16x4(v);
  }
};

// Epilogue for transposed accumulator tiles (see mma_tile_t).  Requires N % 4 == 0 and ldc % 4 == 0.
template <typename T, int TM, int TN, bool OUT_F32>
__device__ __forceinline__ void store_tile_t(const ConvGeom &g, const GemmIO &io, int rep, int mrow0, int ncol0, int lane,
                                             f16v (&acc)[TM][TN]) {
  typedef typename Vec4<T>::type TV;
  const int row_l = lane & 31, h = lane >> 5;
  const float *bias = io.bias ? io.bias + rep * io.bias_rs : nullptr;
  const T *resid = io.resid ? (const T *)io.resid + rep * io.resid_rs : nullptr;
  const T *mask = io.mask ? (const T *)io.mask + rep * io.mask_rs : nullptr;
  const bool bias_vec = (reinterpret_cast<uintptr_t>(bias) & 15) == 0;  // segment offsets need not be 16-byte aligned
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    const int m = mrow0 + tm * 32 + row_l;
    if (m >= g.M) continue;
    const uint32_t pix = row_pixel(g, (uint32_t)m);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int n = ncol0 + tn * 32 + 8 * vg + 4 * h;
        if (n >= g.N) continue;
        const long long o = (long long)pix * io.ldc + n;
        f4 val = {acc[tm][tn][4 * vg], acc[tm][tn][4 * vg + 1], acc[tm][tn][4 * vg + 2], acc[tm][tn][4 * vg + 3]};
        if (bias) {
          if (bias_vec) {
            val += *(const f4 *)(bias + n);
          } else {
            val.x += bias[n], val.y += bias[n + 1], val.z += bias[n + 2], val.w += bias[n + 3];
          }
        }
        if (resid) val += Vec4<T>::to_f32(*(const TV *)(resid + o));
        if (io.relu) {
          val.x = val.x > 0.f ? val.x : 0.f, val.y = val.y > 0.f ? val.y : 0.f;
          val.z = val.z > 0.f ? val.z : 0.f, val.w = val.w > 0.f ? val.w : 0.f;
        }
        if (mask) {
          const f4 mk = Vec4<T>::to_f32(*(const TV *)(mask + o));
          val.x = mk.x > 0.f ? val.x : 0.f, val.y = mk.y > 0.f ? val.y : 0.f;
          val.z = mk.z > 0.f ? val.z : 0.f, val.w = mk.w > 0.f ? val.w : 0.f;
        }
        if (OUT_F32) {
          float *out = (float *)io.out + rep * io.out_rs;
          if (io.accumulate) val += *(const f4 *)(out + o);
          *(f4 *)(out + o) = val;
        } else {
          T *out = (T *)io.out + rep * io.out_rs;
          if (io.accumulate) val += Vec4<T>::to_f32(*(const TV *)(out + o));
          *(TV *)(out + o) = Vec4<T>::from_f32(val);
        }
      }
    }
  }
}

// Epilogue for transposed accumulator tiles, staged through LDS so that global memory sees whole
// rows: each wavefront parks 32 rows x (TN*32) columns of fp32 sums in its own LDS strip, then walks
// the strip in row-major order, four consecutive channels per lane and consecutive lanes on
// consecutive channels -- reads of the residual / mask / old output and the final store all hit
// contiguous runs of a row (the whole row when the tile spans it) instead of 16 bytes per row.
//
// A wavefront issues one vector instruction per four cycles, and with one or two wavefronts per
// SIMD the epilogue is bound by its instruction count, so the walk is kept lean:
//   * lane l handles vectors c = 64*it + l of the strip; (row, channel) of c repeat with period
//     PER = CPR / gcd(64, CPR) in `it`, so PER base offsets are computed once and every vector costs
//     one add (LDS addresses are compile-time offsets from the bases);
//   * global accesses are raw buffer loads / stores: a lane outside the tile gets an offset beyond
//     the buffer and the hardware drops it -- no branches, no 64-bit address arithmetic;
//   * a batch issues all its LDS reads, then all its global reads, then arithmetic and stores, and
//     pays one LDS and one memory latency instead of one per vector.
// Requires N % 4 == 0, ldc % 4 == 0 and M * ldc * 4 < 2^31.  `stage` is this wavefront's strip of
// kStageFloats<TN> floats; the caller has made sure (barrier) that no wavefront still reads LDS
// that it aliases.  A strip is private to its wavefront, whose LDS accesses execute in order: no
// workgroup barrier is needed here.
template <int TN>
constexpr int kStageFloats = 32 * (TN * 32 + 4);

constexpr uint32_t kOobOffset = 0x80000000u;  // beyond any per-replica tensor (each is < 2 GiB)

//
// STAT: column sums of what is stored (the values as rounded to the output type) and of their squares, over the
// wavefront's TM*32 rows: afterwards `wsum[c]` and `wsum[TN*32 + c]`, c < TN*32, hold them for channel ncol0 + c.
// They are the statistics the batch-norm that follows the convolution needs, taken while the tile is at hand
// instead of in a pass of their own over the tensor.  Order of the additions: a lane adds its vectors in walk
// order, then the lanes that share a channel are added in row order - fixed, so the sums are reproducible.
// (`sq_off`: where the squares go relative to the sums; TN*32 unless several wavefronts share a row of sums.)
template <typename T, int TM, int TN, bool OUT_F32, bool STAT = false>
__device__ __forceinline__ void store_tile_lds(const ConvGeom &g, const GemmIO &io, int rep, int mrow0, int ncol0, int lane,
                                               f16v (&acc)[TM][TN], float *stage, float *wsum = nullptr,
                                               int sq_off = TN * 32) {
  typedef unsigned int u2v __attribute__((ext_vector_type(2)));
  constexpr int CW = TN * 32, LD = CW + 4, CPR = CW / 4;
  constexpr int NIT = CPR / 2;                                  // vectors per lane and 32-row strip
  constexpr int PER = CPR % 3 == 0 ? 3 : 1;                     // CPR = 8, 16, 32 divide 64; 24 has period 3
  constexpr int RPP = 64 * PER / CPR;                           // rows per period
  constexpr int BATCH = NIT <= 8 ? NIT : NIT / 2;
  static_assert(NIT % PER == 0 && BATCH % PER == 0 && NIT % BATCH == 0, "walk must split into whole periods");
  constexpr int ES = (int)sizeof(T), OS = OUT_F32 ? 4 : ES;
  const int row_l = lane & 31, h = lane >> 5;
  const uint32_t tensor_elems = (uint32_t)g.M * (uint32_t)io.ldc;
  const __amdgpu_buffer_rsrc_t o_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((char *)io.out + (long long)rep * io.out_rs * OS), 0, (int)(tensor_elems * OS), 0x00020000);
  const __amdgpu_buffer_rsrc_t r_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.resid + rep * io.resid_rs), 0, io.resid ? (int)(tensor_elems * ES) : 0, 0x00020000);
  const __amdgpu_buffer_rsrc_t m_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      (void *)((const T *)io.mask + rep * io.mask_rs), 0, io.mask ? (int)(tensor_elems * ES) : 0, 0x00020000);
  // per lane and phase of the period: strip address, element offset inside a 32-row strip, validity
  int lds_b[PER], row_b[PER], ch_b[PER];
  f4 bias_b[PER];
  f4 sum_b[STAT ? PER : 1], sq_b[STAT ? PER : 1];
#pragma unroll
  for (int r = 0; r < (STAT ? PER : 1); ++r) sum_b[r] = f4{0.f, 0.f, 0.f, 0.f}, sq_b[r] = f4{0.f, 0.f, 0.f, 0.f};
  // what a lane adds for one vector: the stored value (zero outside the tile)
  auto tally = [&](int r, f4 t, uint32_t off) {
    if (off == kOobOffset) t = f4{0.f, 0.f, 0.f, 0.f};
    sum_b[STAT ? r : 0] += t;
    sq_b[STAT ? r : 0] += t * t;
  };
  // stores a vector and, with STAT, adds what was stored to the lane's sums
  auto emit = [&](int r, const f4 &v, uint32_t off) {
    const uint32_t bo = off == kOobOffset ? kOobOffset : off * OS;
    if (OS == 4) {
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, v), o_rsrc, bo, 0, 0);
      if (STAT) tally(r, v, off);
    } else {
      const us4 pk = f32x4_to_bf16x4(v);
      __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u2v, pk), o_rsrc, bo, 0, 0);
      if (STAT) tally(r, Vec4<bf16_t>::to_f32(pk), off);
    }
  };
#pragma unroll
  for (int r = 0; r < PER; ++r) {
    const int c = 64 * r + lane;
    row_b[r] = c / CPR;
    ch_b[r] = (c - row_b[r] * CPR) * 4;
    lds_b[r] = row_b[r] * LD + ch_b[r];
    bias_b[r] = f4{0.f, 0.f, 0.f, 0.f};
    const int n = ncol0 + ch_b[r];
    if (io.bias && n < g.N) {
      const float *bp = io.bias + rep * io.bias_rs + n;   // segment offsets need not be 16-byte aligned
      bias_b[r] = f4{bp[0], bp[1], bp[2], bp[3]};
    }
  }
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");  // the strip has been read out
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const f4 val = {acc[tm][tn][4 * vg], acc[tm][tn][4 * vg + 1], acc[tm][tn][4 * vg + 2], acc[tm][tn][4 * vg + 3]};
        *(f4 *)&stage[row_l * LD + tn * 32 + 8 * vg + 4 * h] = val;
      }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    const int mbase = mrow0 + tm * 32;
#pragma unroll
    for (int b0 = 0; b0 < NIT; b0 += BATCH) {
      f4 val[BATCH], of[BATCH];
      uint32_t off[BATCH];  // element offset, or kOobOffset
      u2v rv[BATCH], mv[BATCH], ov[BATCH];
#pragma unroll
      for (int i = 0; i < BATCH; ++i) {
        const int it = b0 + i, r = it % PER, j = it / PER;
        const int row = row_b[r] + j * RPP, m = mbase + row;
        const bool ok = m < g.M && ncol0 + ch_b[r] < g.N;
        const uint32_t pix = g.plq == 0 ? (uint32_t)m : row_pixel(g, (uint32_t)(ok ? m : 0));
        off[i] = ok ? pix * (uint32_t)io.ldc + (uint32_t)(ncol0 + ch_b[r]) : kOobOffset;
        val[i] = *(const f4 *)&stage[lds_b[r] + j * RPP * LD];
      }
      if (io.resid) {
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
          if (ES == 4) {
            const u4 t = __builtin_amdgcn_raw_buffer_load_b128(r_rsrc, off[i] == kOobOffset ? kOobOffset : off[i] * 4, 0, 0);
            val[i] += __builtin_bit_cast(f4, t);
          } else {
            rv[i] = __builtin_amdgcn_raw_buffer_load_b64(r_rsrc, off[i] == kOobOffset ? kOobOffset : off[i] * 2, 0, 0);
          }
        }
      }
      u4 mv4[ES == 4 ? BATCH : 1];
      if (io.mask) {
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
          if (ES == 4)
            mv4[i] = __builtin_amdgcn_raw_buffer_load_b128(m_rsrc, off[i] == kOobOffset ? kOobOffset : off[i] * 4, 0, 0);
          else
            mv[i] = __builtin_amdgcn_raw_buffer_load_b64(m_rsrc, off[i] == kOobOffset ? kOobOffset : off[i] * 2, 0, 0);
        }
      }
      if (io.accumulate) {
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
          if (OS == 4)
            of[i] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(o_rsrc, off[i] == kOobOffset ? kOobOffset : off[i] * 4, 0, 0));
          else
            ov[i] = __builtin_amdgcn_raw_buffer_load_b64(o_rsrc, off[i] == kOobOffset ? kOobOffset : off[i] * 2, 0, 0);
        }
      }
      if constexpr (PER == 1) {
        // one uniform branch per optional stage and batch, not per vector: a taken branch costs a wavefront
        // tens of cycles of instruction refetch
  #pragma unroll
        for (int i = 0; i < BATCH; ++i) val[i] += bias_b[(b0 + i) % PER];
        if (ES == 2 && io.resid) {
  #pragma unroll
          for (int i = 0; i < BATCH; ++i) val[i] += Vec4<bf16_t>::to_f32(__builtin_bit_cast(us4, rv[i]));
        }
        if (io.relu) {
  #pragma unroll
          for (int i = 0; i < BATCH; ++i) {
            f4 &v = val[i];
            v.x = v.x > 0.f ? v.x : 0.f, v.y = v.y > 0.f ? v.y : 0.f;
            v.z = v.z > 0.f ? v.z : 0.f, v.w = v.w > 0.f ? v.w : 0.f;
          }
        }
        if (io.mask) {
  #pragma unroll
          for (int i = 0; i < BATCH; ++i) {
            f4 &v = val[i];
            const f4 mk = ES == 4 ? __builtin_bit_cast(f4, mv4[ES == 4 ? i : 0]) : Vec4<bf16_t>::to_f32(__builtin_bit_cast(us4, mv[i]));
            v.x = mk.x > 0.f ? v.x : 0.f, v.y = mk.y > 0.f ? v.y : 0.f;
            v.z = mk.z > 0.f ? v.z : 0.f, v.w = mk.w > 0.f ? v.w : 0.f;
          }
        }
        if (io.accumulate) {
  #pragma unroll
          for (int i = 0; i < BATCH; ++i) val[i] += OS == 4 ? of[i] : Vec4<bf16_t>::to_f32(__builtin_bit_cast(us4, ov[i]));
        }
  #pragma unroll
        for (int i = 0; i < BATCH; ++i) emit(0, val[i], off[i]);
      } else {
        // 96-wide tiles (period 3): the per-vector form measured faster there
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
          f4 v = val[i] + bias_b[(b0 + i) % PER];
          if (ES == 2 && io.resid) v += Vec4<bf16_t>::to_f32(__builtin_bit_cast(us4, rv[i]));
          if (io.relu) {
            v.x = v.x > 0.f ? v.x : 0.f, v.y = v.y > 0.f ? v.y : 0.f;
            v.z = v.z > 0.f ? v.z : 0.f, v.w = v.w > 0.f ? v.w : 0.f;
          }
          if (io.mask) {
            const f4 mk = ES == 4 ? __builtin_bit_cast(f4, mv4[ES == 4 ? i : 0]) : Vec4<bf16_t>::to_f32(__builtin_bit_cast(us4, mv[i]));
            v.x = mk.x > 0.f ? v.x : 0.f, v.y = mk.y > 0.f ? v.y : 0.f;
            v.z = mk.z > 0.f ? v.z : 0.f, v.w = mk.w > 0.f ? v.w : 0.f;
          }
          if (io.accumulate) v += OS == 4 ? of[i] : Vec4<bf16_t>::to_f32(__builtin_bit_cast(us4, ov[i]));
          emit((b0 + i) % PER, v, off[i]);
        }
      }
    }
  }
  if (STAT) {
    // lanes that share a channel group sit RPP rows apart in the walk: park the lane sums in the strip (rows
    // 0 .. RPP-1 the sums, RPP .. 2*RPP-1 the squares) and let one lane per group add them
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
    for (int r = 0; r < PER; ++r) {
      *(f4 *)&stage[lds_b[r]] = sum_b[STAT ? r : 0];
      *(f4 *)&stage[RPP * LD + lds_b[r]] = sq_b[STAT ? r : 0];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    if (lane < CPR) {
      f4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < RPP; ++j) a += *(const f4 *)&stage[j * LD + 4 * lane], b += *(const f4 *)&stage[(RPP + j) * LD + 4 * lane];
      *(f4 *)&wsum[4 * lane] = a;
      *(f4 *)&wsum[sq_off + 4 * lane] = b;
    }
  }
}

// Second half of STAT: `wsums` holds, for each of the WAVES_M wavefront rows of a workgroup's tile, BN sums and
// BN sums of squares ([WAVES_M][2][BN] floats, written by store_tile_lds).  They are added in row order and
// written as partial row `prow` of io.stat = [replica][S][2][ldc] doubles, channels n0 .. n0 + BN - 1.
template <int BN, int WAVES_M>
__device__ __forceinline__ void write_tile_sums(const ConvGeom &g, const GemmIO &io, int rep, int S, int prow, int n0,
                                                int tid, const float *wsums) {
  static_assert(2 * BN / 4 <= kThreads, "one thread per vector of sums");
  __syncthreads();
  if (tid < 2 * BN / 4) {
    f4 a = *(const f4 *)&wsums[4 * tid];
#pragma unroll
    for (int w = 1; w < WAVES_M; ++w) a += *(const f4 *)&wsums[w * 2 * BN + 4 * tid];
    const int k = tid >= BN / 4, c = n0 + 4 * (tid - k * (BN / 4));
    if (c < g.N) {
      double *dst = io.stat + (((long long)rep * S + prow) * 2 + k) * io.ldc + c;
      dst[0] = a.x, dst[1] = a.y, dst[2] = a.z, dst[3] = a.w;
    }
  }
}

// Writes a wavefront's TM x TN accumulator tiles: bias, residual, ReLU, mask, accumulate, convert.
template <typename T, int TM, int TN, bool OUT_F32>
__device__ __forceinline__ void store_tile(const ConvGeom &g, const GemmIO &io, int rep, int mrow0, int ncol0, int lane,
                                           f16v (&acc)[TM][TN]) {
  const int col_l = lane & 31, h = lane >> 5;
  const float *bias = io.bias ? io.bias + rep * io.bias_rs : nullptr;
  const T *resid = io.resid ? (const T *)io.resid + rep * io.resid_rs : nullptr;
  const T *mask = io.mask ? (const T *)io.mask + rep * io.mask_rs : nullptr;
#pragma unroll
  for (int tn = 0; tn < TN; ++tn) {
    const int n = ncol0 + tn * 32 + col_l;
    if (n >= g.N) continue;
    const float bv = bias ? bias[n] : 0.f;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = mrow0 + tm * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (m >= g.M) continue;
        const long long o = (long long)m * io.ldc + n;
        float val = acc[tm][tn][v] + bv;
        if (resid) val += to_f32<T>(resid[o]);
        if (io.relu) val = val > 0.f ? val : 0.f;
        if (mask) val = to_f32<T>(mask[o]) > 0.f ? val : 0.f;
        if (OUT_F32) {
          float *out = (float *)io.out + rep * io.out_rs;
          if (io.accumulate) val += out[o];
          out[o] = val;
        } else {
          T *out = (T *)io.out + rep * io.out_rs;
          if (io.accumulate) val += to_f32<T>(out[o]);
          out[o] = from_f32<T>(val);
        }
      }
    }
  }
}

}  // namespace igemm_dev
