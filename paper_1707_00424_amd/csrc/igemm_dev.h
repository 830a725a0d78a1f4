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
// Requires N % 4 == 0 and ldc % 4 == 0.  `stage` is this wavefront's strip of kStageFloats<TN>
// floats; the caller has made sure (barrier) that no wavefront still reads LDS that it aliases.
// Every wavefront of the workgroup must call this (it contains workgroup barriers).
template <int TN>
constexpr int kStageFloats = 32 * (TN * 32 + 4);

template <typename T, int TM, int TN, bool OUT_F32>
__device__ __forceinline__ void store_tile_lds(const ConvGeom &g, const GemmIO &io, int rep, int mrow0, int ncol0, int lane,
                                               f16v (&acc)[TM][TN], float *stage) {
  typedef typename Vec4<T>::type TV;
  constexpr int CW = TN * 32, LD = CW + 4, CPR = CW / 4;
  const int row_l = lane & 31, h = lane >> 5;
  const float *bias = io.bias ? io.bias + rep * io.bias_rs : nullptr;
  const T *resid = io.resid ? (const T *)io.resid + rep * io.resid_rs : nullptr;
  const T *mask = io.mask ? (const T *)io.mask + rep * io.mask_rs : nullptr;
  const bool bias_vec = (reinterpret_cast<uintptr_t>(bias) & 15) == 0;  // segment offsets need not be 16-byte aligned
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    if (tm) __syncthreads();  // the strip has been read out
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const f4 val = {acc[tm][tn][4 * vg], acc[tm][tn][4 * vg + 1], acc[tm][tn][4 * vg + 2], acc[tm][tn][4 * vg + 3]};
        *(f4 *)&stage[row_l * LD + tn * 32 + 8 * vg + 4 * h] = val;
      }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < CPR / 2; ++it) {
      const int c = it * 64 + lane;
      const int row = c / CPR, ch = (c - row * CPR) * 4;
      const int m = mrow0 + tm * 32 + row, n = ncol0 + ch;
      if (m >= g.M || n >= g.N) continue;
      const long long o = (long long)row_pixel(g, (uint32_t)m) * io.ldc + n;
      f4 val = *(const f4 *)&stage[row * LD + ch];
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
