// Memory-bound kernels of the Parle step: fused inner update (8a)+(8b), replica mean (8d),
// fused outer update (8c) + reset, ensemble spread.  Every tensor is streamed once with 16-byte
// accesses; nothing is reused, so loads and stores are non-temporal.
#include <stdlib.h>

#include <mutex>
#include <string>

#include "common.h"

namespace {

constexpr int kThreads = 256;

struct Tuning {
  int inner_unroll;   // float4 per thread per trip
  int blocks_per_cu;  // 0 = one trip per thread (grid covers the tensor)
  int nontemporal;
  int contiguous;     // 1: a block's U vectors per thread are adjacent 4 KiB chunks; 0: a grid stride apart
};

const Tuning &tuning() {
  static Tuning t = [] {
    Tuning v{4, 0, 1, 1};
    if (const char *s = getenv("PARLE_UPD_CONTIG")) v.contiguous = atoi(s);
    if (const char *s = getenv("PARLE_UPD_UNROLL")) v.inner_unroll = atoi(s);
    if (const char *s = getenv("PARLE_UPD_BLOCKS_PER_CU")) v.blocks_per_cu = atoi(s);
    if (const char *s = getenv("PARLE_UPD_NT")) v.nontemporal = atoi(s);
    return v;
  }();
  return t;
}

template <bool NT>
__device__ __forceinline__ f4 ld4(const f4 *p) {
  if (NT) return __builtin_nontemporal_load(p);
  return *p;
}
template <bool NT>
__device__ __forceinline__ void st4(f4 *p, f4 v) {
  if (NT)
    __builtin_nontemporal_store(v, p);
  else
    *p = v;
}
__device__ __forceinline__ us4 to_bf16x4(f4 v) {
  return f32x4_to_bf16x4(v);
}

// ---------------------------------------------------------------------------------------------
// (8a) with Nesterov momentum, then (8b).  One flat pass over n*n_pad elements.
// ---------------------------------------------------------------------------------------------
template <int U, bool NT, bool BF>
__global__ __launch_bounds__(kThreads) void k_inner_update(const f4 *__restrict__ G, const f4 *__restrict__ X,
                                                           f4 *__restrict__ Y, f4 *__restrict__ VY,
                                                           f4 *__restrict__ Z, us4 *__restrict__ Y16, int64_t n4,
                                                           float eta, float mu, float alpha, float wd, float g_arg,
                                                           const float *__restrict__ coupling, int contiguous) {
  // a captured launch cannot change its arguments: it reads the proximal multiplier from memory
  const float g = coupling ? coupling[0] : g_arg;
  // contiguous: block b owns vectors [b*U*256, (b+1)*U*256); else vector u of a thread is a grid stride away
  const int64_t stride = contiguous ? kThreads : (int64_t)gridDim.x * kThreads;
  const int64_t first = contiguous ? (int64_t)blockIdx.x * kThreads * U + threadIdx.x
                                   : (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t trip = (int64_t)gridDim.x * kThreads * U;
  const float one_m_alpha = 1.0f - alpha;
  for (int64_t q0 = first; q0 < n4; q0 += trip) {
    f4 gr[U], x[U], y[U], v[U], z[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * stride;
      if (q < n4) {
        gr[u] = ld4<NT>(G + q);
        x[u] = ld4<NT>(X + q);
        y[u] = ld4<NT>(Y + q);
        v[u] = ld4<NT>(VY + q);
        z[u] = ld4<NT>(Z + q);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * stride;
      if (q < n4) {
        const f4 d = gr[u] + wd * y[u] + g * (y[u] - x[u]);
        const f4 vn = mu * v[u] + d;
        const f4 yn = y[u] - eta * (d + mu * vn);
        const f4 zn = alpha * z[u] + one_m_alpha * yn;
        st4<NT>(VY + q, vn);
        st4<NT>(Y + q, yn);
        st4<NT>(Z + q, zn);
        if (BF) __builtin_nontemporal_store(to_bf16x4(yn), Y16 + q);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Plain streams with the access shape of the update kernels and no arithmetic to speak of: R arrays
// read, W arrays written, 16 bytes per lane, four vectors in flight per array.  What this reaches is
// what the memory system gives that mix of reads and writes; the update kernels are measured against it.
// ---------------------------------------------------------------------------------------------
template <int R, int W>
__global__ __launch_bounds__(kThreads) void k_stream(const f4 *__restrict__ src, f4 *__restrict__ dst, int64_t n4) {
  constexpr int U = 4;
  const int64_t trip = (int64_t)gridDim.x * kThreads * U;
  f4 keep = {0.f, 0.f, 0.f, 0.f};
  for (int64_t q0 = (int64_t)blockIdx.x * kThreads * U + threadIdx.x; q0 < n4; q0 += trip) {
    f4 v[R > 0 ? R : 1][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * kThreads;
#pragma unroll
      for (int r = 0; r < R; ++r) v[r][u] = q < n4 ? ld4<true>(src + r * n4 + q) : keep;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * kThreads;
      f4 s = {1.f, 2.f, 3.f, 4.f};
#pragma unroll
      for (int r = 0; r < R; ++r) s += v[r][u];
      if (W == 0) keep += s;
#pragma unroll
      for (int w = 0; w < W; ++w)
        if (q < n4) st4<true>(dst + w * n4 + q, s);
    }
  }
  // read-only: the loads must stay live; a sum of finite inputs never takes this value
  if (W == 0 && keep.x + keep.y + keep.z + keep.w == __builtin_inff()) dst[0] = keep;
}

// ---------------------------------------------------------------------------------------------
// (8d) with eta'' = rho/n: column mean of the stacked replicas, summed in replica order.
// ---------------------------------------------------------------------------------------------
// N > 0: compile-time replica count, all N x U loads of a thread issued before the first add; a block owns U
// adjacent 4 KiB chunks of every row.  N = 0: any n, one load at a time.
template <int N, int U, bool NT>
__global__ __launch_bounds__(kThreads) void k_replica_mean(const f4 *__restrict__ X, f4 *__restrict__ XR, int n,
                                                           int64_t np4) {
  const float fn = (float)(N > 0 ? N : n);
  if (N == 0) {
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < np4; q += stride) {
      f4 s = ld4<NT>(X + q);
      for (int a = 1; a < n; ++a) s += ld4<NT>(X + (int64_t)a * np4 + q);
      XR[q] = s / fn;  // kept cacheable: the outer update reads it right away
    }
    return;
  }
  const int64_t trip = (int64_t)gridDim.x * kThreads * U;
  for (int64_t q0 = (int64_t)blockIdx.x * kThreads * U + threadIdx.x; q0 < np4; q0 += trip) {
    f4 xs[N > 0 ? N : 1][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * kThreads;
#pragma unroll
      for (int a = 0; a < N; ++a)
        if (q < np4) xs[a][u] = ld4<NT>(X + (int64_t)a * np4 + q);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * kThreads;
      if (q < np4) {
        f4 s = xs[0][u];
#pragma unroll
        for (int a = 1; a < N; ++a) s += xs[a][u];   // replica order, as the one-at-a-time form
        XR[q] = s / fn;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// (8c) with Nesterov momentum and the reset of y (z, vy per flags).  blockIdx.y = replica.
// ---------------------------------------------------------------------------------------------
template <bool NT, bool BF>
__global__ __launch_bounds__(kThreads) void k_outer_update(f4 *__restrict__ X, f4 *__restrict__ Z,
                                                           f4 *__restrict__ VX, f4 *__restrict__ Y,
                                                           f4 *__restrict__ VY, const f4 *__restrict__ XR,
                                                           us4 *__restrict__ Y16, int64_t np4, float eta, float mu,
                                                           float cz, float r, int reset_flags) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  const int64_t base = (int64_t)blockIdx.y * np4;
  const f4 zero = {0.f, 0.f, 0.f, 0.f};
  for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < np4; q += stride) {
    const f4 x = ld4<NT>(X + base + q);
    const f4 z = ld4<NT>(Z + base + q);
    const f4 v = ld4<NT>(VX + base + q);
    const f4 xr = XR[q];
    const f4 d = cz * (x - z) + r * (x - xr);
    const f4 vn = mu * v + d;
    const f4 xn = x - eta * (d + mu * vn);
    st4<NT>(VX + base + q, vn);
    st4<NT>(X + base + q, xn);
    st4<NT>(Y + base + q, xn);
    if (reset_flags & 1) st4<NT>(Z + base + q, xn);
    if (reset_flags & 2) st4<NT>(VY + base + q, zero);
    if (BF) __builtin_nontemporal_store(to_bf16x4(xn), Y16 + base + q);
  }
}

// Same update with the replica mean formed in registers: every x^a[i] is read once, the mean is
// written to x_ref, and no second pass over x is needed.  N > 0: compile-time replica count; the N loads
// of x are issued together, z^a and v^a are fetched per replica as its update is formed (holding all
// 3N vectors costs a wavefront of occupancy and gains nothing).
template <int N, int U, bool NT, bool BF>
__global__ __launch_bounds__(kThreads) void k_outer_fused(f4 *__restrict__ X, f4 *__restrict__ Z, f4 *__restrict__ VX,
                                                          f4 *__restrict__ Y, f4 *__restrict__ VY,
                                                          f4 *__restrict__ XR, us4 *__restrict__ Y16, int n_rt,
                                                          int64_t np4, float eta, float mu, float cz, float r,
                                                          int reset_flags, int lagged) {
  const f4 zero = {0.f, 0.f, 0.f, 0.f};
  const int n = N > 0 ? N : n_rt;
  const float fn = (float)n;
  // a block owns U adjacent 4 KiB chunks of every row
  const int64_t trip = (int64_t)gridDim.x * kThreads * U;
  for (int64_t q0 = (int64_t)blockIdx.x * kThreads * U + threadIdx.x; q0 < np4; q0 += trip) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t q = q0 + u * kThreads;
      if (q >= np4) break;
      f4 xs[N > 0 ? N : 1];
      f4 s;
      if (N > 0) {
#pragma unroll
        for (int a = 0; a < N; ++a) xs[a] = ld4<NT>(X + (int64_t)a * np4 + q);
        s = xs[0];
#pragma unroll
        for (int a = 1; a < N; ++a) s += xs[a];
      } else {
        s = X[q];
        for (int a = 1; a < n; ++a) s += X[(int64_t)a * np4 + q];
      }
      const f4 mean = s / fn;
      const f4 xr = lagged ? XR[q] : mean;
      st4<NT>(XR + q, mean);
#pragma unroll
      for (int a = 0; a < n; ++a) {
        const int64_t o = (int64_t)a * np4 + q;
        const f4 x = N > 0 ? xs[N > 0 ? a : 0] : X[o];
        const f4 z = ld4<NT>(Z + o);
        const f4 v = ld4<NT>(VX + o);
        const f4 d = cz * (x - z) + r * (x - xr);
        const f4 vn = mu * v + d;
        const f4 xn = x - eta * (d + mu * vn);
        st4<NT>(VX + o, vn);
        st4<NT>(X + o, xn);
        st4<NT>(Y + o, xn);
        if (reset_flags & 1) st4<NT>(Z + o, xn);
        if (reset_flags & 2) st4<NT>(VY + o, zero);
        if (BF) __builtin_nontemporal_store(to_bf16x4(xn), Y16 + o);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Elastic-SGD (Section 2.2), both coupled updates in one pass over a column:
//   x^a <- x^a - eta [ grad + wd x^a + r (x^a - x) ]   (Nesterov momentum on the replicas)
//   x   <- x - eta_ref ( x - mean_a x^a )               (mean of the replicas before the move)
// ---------------------------------------------------------------------------------------------
template <int N, bool BF>
__global__ __launch_bounds__(kThreads) void k_elastic_step(const f4 *__restrict__ G, f4 *__restrict__ XA,
                                                           f4 *__restrict__ V, f4 *__restrict__ XR,
                                                           us4 *__restrict__ X16, int n_rt, int64_t np4, float eta,
                                                           float eta_ref, float mu, float wd, float r_arg,
                                                           const float *__restrict__ coupling) {
  const float r = coupling ? coupling[1] : r_arg;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  const int n = N > 0 ? N : n_rt;
  const float fn = (float)n;
  for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < np4; q += stride) {
    const f4 xr = XR[q];
    f4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int a = 0; a < n; ++a) {
      const int64_t o = (int64_t)a * np4 + q;
      const f4 x = ld4<true>(XA + o);
      const f4 gr = ld4<true>(G + o);
      const f4 v = ld4<true>(V + o);
      s = a ? s + x : x;
      const f4 d = gr + wd * x + r * (x - xr);
      const f4 vn = mu * v + d;
      const f4 xn = x - eta * (d + mu * vn);
      st4<true>(V + o, vn);
      st4<true>(XA + o, xn);
      if (BF) __builtin_nontemporal_store(to_bf16x4(xn), X16 + o);
    }
    XR[q] = xr - eta_ref * (xr - s / fn);
  }
}

__global__ void k_set_coupling(float *dst, float g, float r) {
  if (threadIdx.x == 0 && blockIdx.x == 0) dst[0] = g, dst[1] = r;
}

// ---------------------------------------------------------------------------------------------
// sum_a ||x^a - x_ref||^2: per-thread fp32 partial over a few elements, fp64 from the wavefront
// reduction on; per-block partials are summed by one block in a fixed order (deterministic).
// ---------------------------------------------------------------------------------------------
constexpr int kSpreadBlocks = 4096;

// Scratch of the entry point that allocates nothing: the per-workgroup partial sums of one spread launch,
// 32 KiB per GPU, held until the process ends.  In host code this name is only a stand-in for the symbol:
// the device address is fetched once per device (static_spread_scratch below) and that pointer is what
// kernels receive.
static __device__ __align__(256) double scratch[kSpreadBlocks];

__global__ __launch_bounds__(kThreads) void k_spread_partial(const f4 *__restrict__ X, const f4 *__restrict__ XR,
                                                             int n, int64_t np4, double *__restrict__ partial) {
  __shared__ double lds[kThreads / PARLE_WAVE];
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  double acc = 0.0;
  for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < np4; q += stride) {
    const f4 xr = XR[q];
    float part = 0.f;
    for (int a = 0; a < n; ++a) {
      const f4 d = X[(int64_t)a * np4 + q] - xr;
      part += d.x * d.x + d.y * d.y + d.z * d.z + d.w * d.w;
    }
    acc += (double)part;
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & (PARLE_WAVE - 1)) == 0) lds[threadIdx.x / PARLE_WAVE] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int w = 0; w < kThreads / PARLE_WAVE; ++w) s += lds[w];
    partial[blockIdx.x] = s;
  }
}

__global__ __launch_bounds__(kThreads) void k_spread_final(const double *__restrict__ partial, int count,
                                                           float *__restrict__ out) {
  __shared__ double lds[kThreads / PARLE_WAVE];
  double acc = 0.0;
  for (int i = threadIdx.x; i < count; i += kThreads) acc += partial[i];
  acc = wave_sum(acc);
  if ((threadIdx.x & (PARLE_WAVE - 1)) == 0) lds[threadIdx.x / PARLE_WAVE] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int w = 0; w < kThreads / PARLE_WAVE; ++w) s += lds[w];
    out[0] = (float)s;
  }
}

int num_cus() {
  static int cus = [] {
    int dev = 0, v = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
      int q = 0;
      if (hipDeviceGetAttribute(&q, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && q > 0) v = q;
    }
    return v;
  }();
  return cus;
}

int grid_for(int64_t items, int per_thread_trip) {
  const Tuning &t = tuning();
  int64_t need = (items + (int64_t)kThreads * per_thread_trip - 1) / ((int64_t)kThreads * per_thread_trip);
  if (need < 1) need = 1;
  if (t.blocks_per_cu > 0) {
    const int64_t cap = (int64_t)num_cus() * t.blocks_per_cu;
    if (need > cap) need = cap;
  }
  if (need > 0x7fffffff) need = 0x7fffffff;
  return (int)need;
}

// vectors per thread and row of the replica mean and the fused outer update (PARLE_OUTER_UNROLL = 1 or 2)
int outer_unroll() {
  static int u = [] {
    const char *s = getenv("PARLE_OUTER_UNROLL");
    const int v = s ? atoi(s) : 1;
    return v == 2 ? 2 : 1;
  }();
  return u;
}

parle_status check_flat_args(int32_t n, int64_t n_pad) {
  if (n < 1 || n_pad < 4 || (n_pad & 3)) return PARLE_EINVAL;
  if ((double)n * (double)n_pad >= 1099511627776.0) return PARLE_ESIZE;
  return PARLE_OK;
}

parle_status launched() { return hipGetLastError() == hipSuccess ? PARLE_OK : PARLE_EHIP; }

}  // namespace

namespace {
__global__ __launch_bounds__(kThreads) void k_to_bf16(const f4 *__restrict__ src, us4 *__restrict__ dst, int64_t n4) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < n4; q += stride) dst[q] = to_bf16x4(src[q]);
}
}  // namespace

parle_status parle_internal_to_bf16(hipStream_t st, const float *src, void *dst, int64_t count) {
  if (count < 4 || (count & 3) || !src || !dst) return PARLE_EINVAL;
  const int64_t n4 = count / 4;
  hipLaunchKernelGGL(k_to_bf16, dim3(grid_for(n4, 1)), dim3(kThreads), 0, st, (const f4 *)src, (us4 *)dst, n4);
  return launched();
}

__global__ void k_set_step(long long *dst, long long k, int add) {
  if (threadIdx.x == 0 && blockIdx.x == 0) dst[0] = add ? dst[0] + 1 : k;
}

parle_status parle_internal_set_step(hipStream_t st, long long *step_dev, long long k) {
  if (!step_dev) return PARLE_EINVAL;
  hipLaunchKernelGGL(k_set_step, dim3(1), dim3(64), 0, st, step_dev, k, 0);
  return launched();
}
parle_status parle_internal_advance_step(hipStream_t st, long long *step_dev) {
  if (!step_dev) return PARLE_EINVAL;
  hipLaunchKernelGGL(k_set_step, dim3(1), dim3(64), 0, st, step_dev, 0LL, 1);
  return launched();
}

parle_status parle_internal_set_coupling(hipStream_t st, float *coupling_dev, float g, float r) {
  if (!coupling_dev) return PARLE_EINVAL;
  hipLaunchKernelGGL(k_set_coupling, dim3(1), dim3(64), 0, st, coupling_dev, g, r);
  return launched();
}

parle_status parle_internal_inner_update(hipStream_t st, int32_t n, int64_t n_pad, const float *grad, const float *x,
                                         float *y, float *vy, float *z, void *y_bf16, float eta_inner, float momentum,
                                         float alpha, float weight_decay, float g, const float *coupling_dev) {
  if (parle_status s = check_flat_args(n, n_pad)) return s;
  if (!grad || !x || !y || !vy || !z) return PARLE_EINVAL;
  if (!aligned_to(grad, 16) || !aligned_to(x, 16) || !aligned_to(y, 16) || !aligned_to(vy, 16) || !aligned_to(z, 16) ||
      !aligned_to(y_bf16, 8))
    return PARLE_EALIGN;
  const int64_t n4 = (int64_t)n * n_pad / 4;
  const Tuning &t = tuning();
#define LAUNCH_INNER(U, NT, BF)                                                                                   \
  hipLaunchKernelGGL((k_inner_update<U, NT, BF>), dim3(grid_for(n4, U)), dim3(kThreads), 0, st, (const f4 *)grad, \
                     (const f4 *)x, (f4 *)y, (f4 *)vy, (f4 *)z, (us4 *)y_bf16, n4, eta_inner, momentum, alpha,    \
                     weight_decay, g, coupling_dev, t.contiguous)
#define PICK_INNER(U)                   \
  do {                                  \
    if (t.nontemporal) {                \
      if (y_bf16)                       \
        LAUNCH_INNER(U, true, true);    \
      else                              \
        LAUNCH_INNER(U, true, false);   \
    } else {                            \
      if (y_bf16)                       \
        LAUNCH_INNER(U, false, true);   \
      else                              \
        LAUNCH_INNER(U, false, false);  \
    }                                   \
  } while (0)
  switch (t.inner_unroll) {
    case 1: PICK_INNER(1); break;
    case 2: PICK_INNER(2); break;
    case 8: PICK_INNER(8); break;
    default: PICK_INNER(4); break;
  }
#undef PICK_INNER
#undef LAUNCH_INNER
  return launched();
}

parle_status parle_internal_elastic_step(hipStream_t st, int32_t n, int64_t n_pad, const float *grad, float *xa,
                                         float *v, float *x_ref, void *xa_bf16, float eta, float eta_ref,
                                         float momentum, float weight_decay, float r, const float *coupling_dev) {
  if (parle_status s = check_flat_args(n, n_pad)) return s;
  if (!grad || !xa || !v || !x_ref) return PARLE_EINVAL;
  if (!aligned_to(grad, 16) || !aligned_to(xa, 16) || !aligned_to(v, 16) || !aligned_to(x_ref, 16) ||
      !aligned_to(xa_bf16, 8))
    return PARLE_EALIGN;
  const int64_t np4 = n_pad / 4;
  dim3 grid(grid_for(np4, 1));
#define LAUNCH_ELASTIC(N, BF)                                                                                     \
  hipLaunchKernelGGL((k_elastic_step<N, BF>), grid, dim3(kThreads), 0, st, (const f4 *)grad, (f4 *)xa, (f4 *)v,    \
                     (f4 *)x_ref, (us4 *)xa_bf16, n, np4, eta, eta_ref, momentum, weight_decay, r, coupling_dev)
#define PICK_ELASTIC(N)                                                    \
  case N:                                                                  \
    if (xa_bf16) LAUNCH_ELASTIC(N, true); else LAUNCH_ELASTIC(N, false);   \
    break
  switch (n) {
    PICK_ELASTIC(1);
    PICK_ELASTIC(2);
    PICK_ELASTIC(3);
    PICK_ELASTIC(4);
    PICK_ELASTIC(5);
    PICK_ELASTIC(6);
    PICK_ELASTIC(7);
    PICK_ELASTIC(8);
    default:
      if (xa_bf16) LAUNCH_ELASTIC(0, true); else LAUNCH_ELASTIC(0, false);
      break;
  }
#undef PICK_ELASTIC
#undef LAUNCH_ELASTIC
  return launched();
}

extern "C" {

parle_status parle_k_inner_update(void *hip_stream, int32_t n, int64_t n_pad, const float *grad, const float *x,
                                  float *y, float *vy, float *z, void *y_bf16, float eta_inner, float momentum,
                                  float alpha, float weight_decay, float g) {
  return parle_internal_inner_update((hipStream_t)hip_stream, n, n_pad, grad, x, y, vy, z, y_bf16, eta_inner, momentum,
                                     alpha, weight_decay, g, nullptr);
}

parle_status parle_k_elastic_step(void *hip_stream, int32_t n, int64_t n_pad, const float *grad, float *xa, float *v,
                                  float *x_ref, void *xa_bf16, float eta, float eta_ref, float momentum,
                                  float weight_decay, float r) {
  return parle_internal_elastic_step((hipStream_t)hip_stream, n, n_pad, grad, xa, v, x_ref, xa_bf16, eta, eta_ref,
                                     momentum, weight_decay, r, nullptr);
}

parle_status parle_k_replica_mean(void *hip_stream, int32_t n, int64_t n_pad, const float *x, float *x_ref) {
  if (parle_status s = check_flat_args(n, n_pad)) return s;
  if (!x || !x_ref) return PARLE_EINVAL;
  if (!aligned_to(x, 16) || !aligned_to(x_ref, 16)) return PARLE_EALIGN;
  const int64_t np4 = n_pad / 4;
  hipStream_t st = (hipStream_t)hip_stream;
  const int U = outer_unroll();
#define LAUNCH_MEAN(N, UU)                                                                                          \
  hipLaunchKernelGGL((k_replica_mean<N, UU, true>), dim3(grid_for(np4, UU)), dim3(kThreads), 0, st, (const f4 *)x, \
                     (f4 *)x_ref, n, np4)
#define PICK_MEAN(N)           \
  case N:                      \
    if (U == 2)                \
      LAUNCH_MEAN(N, 2);       \
    else                       \
      LAUNCH_MEAN(N, 1);       \
    break
  switch (n) {
    PICK_MEAN(1);
    PICK_MEAN(2);
    PICK_MEAN(3);
    PICK_MEAN(4);
    PICK_MEAN(5);
    PICK_MEAN(6);
    PICK_MEAN(7);
    PICK_MEAN(8);
    default: LAUNCH_MEAN(0, 1); break;
  }
#undef PICK_MEAN
#undef LAUNCH_MEAN
  return launched();
}

parle_status parle_k_outer_update(void *hip_stream, int32_t n, int64_t n_pad, float *x, float *z, float *vx,
                                  float *y, float *vy, float *x_ref, void *y_bf16, float eta_outer, float momentum,
                                  float c_z, float r, int32_t reset_flags, int32_t fuse_mean, int32_t lagged) {
  if (parle_status s = check_flat_args(n, n_pad)) return s;
  if (!x || !z || !vx || !y || !vy || !x_ref) return PARLE_EINVAL;
  if (n > 65535) return PARLE_ESIZE;
  if (!aligned_to(x, 16) || !aligned_to(z, 16) || !aligned_to(vx, 16) || !aligned_to(y, 16) || !aligned_to(vy, 16) ||
      !aligned_to(x_ref, 16) || !aligned_to(y_bf16, 8))
    return PARLE_EALIGN;
  if (lagged && !fuse_mean) return PARLE_EINVAL;  // the unfused path takes whatever x_ref holds
  const int64_t np4 = n_pad / 4;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool nt = tuning().nontemporal != 0;
  if (!fuse_mean) {
    dim3 grid(grid_for(np4, 1), n);
#define LAUNCH_OUTER(NT, BF)                                                                                       \
  hipLaunchKernelGGL((k_outer_update<NT, BF>), grid, dim3(kThreads), 0, st, (f4 *)x, (f4 *)z, (f4 *)vx, (f4 *)y,   \
                     (f4 *)vy, (const f4 *)x_ref, (us4 *)y_bf16, np4, eta_outer, momentum, c_z, r, reset_flags)
    if (nt) {
      if (y_bf16) LAUNCH_OUTER(true, true); else LAUNCH_OUTER(true, false);
    } else {
      if (y_bf16) LAUNCH_OUTER(false, true); else LAUNCH_OUTER(false, false);
    }
#undef LAUNCH_OUTER
    return launched();
  }
  const int U = outer_unroll();
#define LAUNCH_FUSED_U(N, UU, BF)                                                                                       \
  hipLaunchKernelGGL((k_outer_fused<N, UU, true, BF>), dim3(grid_for(np4, UU)), dim3(kThreads), 0, st, (f4 *)x, (f4 *)z, \
                     (f4 *)vx, (f4 *)y, (f4 *)vy, (f4 *)x_ref, (us4 *)y_bf16, n, np4, eta_outer, momentum, c_z, r,       \
                     reset_flags, lagged)
#define LAUNCH_FUSED(N, BF)       \
  do {                            \
    if (U == 2 && N > 0)          \
      LAUNCH_FUSED_U(N, 2, BF);   \
    else                          \
      LAUNCH_FUSED_U(N, 1, BF);   \
  } while (0)
#define PICK_FUSED(N)                                               \
  case N:                                                           \
    if (y_bf16) LAUNCH_FUSED(N, true); else LAUNCH_FUSED(N, false); \
    break
  switch (n) {
    PICK_FUSED(1);
    PICK_FUSED(2);
    PICK_FUSED(3);
    PICK_FUSED(4);
    PICK_FUSED(5);
    PICK_FUSED(6);
    PICK_FUSED(7);
    PICK_FUSED(8);
    default:
      if (y_bf16) LAUNCH_FUSED(0, true); else LAUNCH_FUSED(0, false);
      break;
  }
#undef PICK_FUSED
#undef LAUNCH_FUSED
#undef LAUNCH_FUSED_U
  return launched();
}

parle_status parle_k_spread(void *hip_stream, int32_t n, int64_t n_pad, const float *x, const float *x_ref,
                            double *partial_dev, float *out_dev) {
  if (parle_status s = check_flat_args(n, n_pad)) return s;
  if (!x || !x_ref || !partial_dev || !out_dev) return PARLE_EINVAL;
  if (!aligned_to(x, 16) || !aligned_to(x_ref, 16) || !aligned_to(partial_dev, 8)) return PARLE_EALIGN;
  const int64_t np4 = n_pad / 4;
  int64_t blocks = (np4 + kThreads - 1) / kThreads;
  if (blocks > kSpreadBlocks) blocks = kSpreadBlocks;
  hipStream_t st = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(k_spread_partial, dim3((int)blocks), dim3(kThreads), 0, st, (const f4 *)x, (const f4 *)x_ref, n,
                     np4, partial_dev);
  hipLaunchKernelGGL(k_spread_final, dim3(1), dim3(kThreads), 0, st, (const double *)partial_dev, (int)blocks, out_dev);
  return launched();
}

parle_status parle_k_stream_reference(void *hip_stream, int32_t reads, int32_t writes, int64_t count,
                                      const float *src_dev, float *dst_dev) {
  if (count < 4 || count % 4 || count > (1LL << 40)) return PARLE_ESIZE;
  if (!dst_dev || (reads > 0 && !src_dev)) return PARLE_EINVAL;
  if (!aligned_to(src_dev, 16) || !aligned_to(dst_dev, 16)) return PARLE_EALIGN;
  const int64_t n4 = count / 4;
  const dim3 grid(grid_for(n4, 4));
  hipStream_t st = (hipStream_t)hip_stream;
  const f4 *src = (const f4 *)src_dev;
  f4 *dst = (f4 *)dst_dev;
  if (reads == 1 && writes == 0)
    hipLaunchKernelGGL((k_stream<1, 0>), grid, dim3(kThreads), 0, st, src, dst, n4);
  else if (reads == 0 && writes == 1)
    hipLaunchKernelGGL((k_stream<0, 1>), grid, dim3(kThreads), 0, st, src, dst, n4);
  else if (reads == 1 && writes == 1)
    hipLaunchKernelGGL((k_stream<1, 1>), grid, dim3(kThreads), 0, st, src, dst, n4);
  else if (reads == 5 && writes == 3)
    hipLaunchKernelGGL((k_stream<5, 3>), grid, dim3(kThreads), 0, st, src, dst, n4);
  else
    return PARLE_EINVAL;
  return launched();
}

}  // extern "C"

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
double *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (every GPU holds its own copy of the array).
parle_status static_spread_scratch(double **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    parle_internal_set_error("parle_k_spread_static: no current HIP device (or device index >= 64)");
    return PARLE_EHIP;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      parle_internal_set_error(std::string("parle_k_spread_static: hipGetSymbolAddress failed: ") + hipGetErrorString(e));
      return PARLE_EHIP;
    }
    g_scratch_ptr[dev] = (double *)p;
  }
  *out = g_scratch_ptr[dev];
  return PARLE_OK;
}
}  // namespace

extern "C" parle_status parle_k_spread_static(void *hip_stream, int32_t n, int64_t n_pad, const float *x,
                                              const float *x_ref, float *out_dev) {
  if (n < 1 || n_pad < 4 || (n_pad & 3) || !x || !x_ref || !out_dev) {
    parle_internal_set_error("parle_k_spread_static: n >= 1, n_pad a positive multiple of 4 and non-null pointers needed");
    return PARLE_EINVAL;
  }
  if ((double)n * (double)n_pad > (double)PARLE_SPREAD_STATIC_MAX_ELEMS) {
    parle_internal_set_error("parle_k_spread_static: n * n_pad exceeds PARLE_SPREAD_STATIC_MAX_ELEMS (2^34); use "
                             "parle_k_spread with a scratch buffer of the caller's");
    return PARLE_ESIZE;
  }
  if (!aligned_to(x, 16) || !aligned_to(x_ref, 16)) {
    parle_internal_set_error("parle_k_spread_static: x and x_ref must be 16-byte aligned");
    return PARLE_EALIGN;
  }
  double *partial = nullptr;
  if (parle_status s = static_spread_scratch(&partial)) return s;
  // every slot the second kernel reads is written by the first one of the same call: nothing to clear
  return parle_k_spread(hip_stream, n, n_pad, x, x_ref, partial, out_dev);
}
