// Memory-bound layer kernels: loss, pooling, batch normalisation, bias gradients, weight transposes.
// All reductions use a fixed order (per-thread serial, wavefront shuffle, serial over wavefronts and
// over row-splits), so results are bit-reproducible from run to run.
#include "nn.h"

namespace {

constexpr int kThreads = 256;
constexpr float kBnEps = 1e-5f;
constexpr float kBnMomentum = 0.1f;

template <typename T>
__device__ __forceinline__ float ldf(const T *p, long long i);
template <>
__device__ __forceinline__ float ldf<float>(const float *p, long long i) {
  return p[i];
}
template <>
__device__ __forceinline__ float ldf<bf16_t>(const bf16_t *p, long long i) {
  return bf16_to_f32(p[i]);
}
template <typename T>
__device__ __forceinline__ void stf(T *p, long long i, float v);
template <>
__device__ __forceinline__ void stf<float>(float *p, long long i, float v) {
  p[i] = v;
}
template <>
__device__ __forceinline__ void stf<bf16_t>(bf16_t *p, long long i, float v) {
  p[i] = f32_to_bf16(v);
}

inline int blocks_for(long long items, int cap = 65535 * 16) {
  long long b = (items + kThreads - 1) / kThreads;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (int)b;
}

// ------------------------------------------------------------------ softmax cross-entropy
template <typename T>
__global__ __launch_bounds__(kThreads) void k_softmax_train(int B, int C, const float *__restrict__ logits,
                                                            long long logits_rs, const int32_t *__restrict__ labels,
                                                            float *__restrict__ loss_out, T *__restrict__ dl,
                                                            long long dl_rs) {
  __shared__ float red[kThreads / PARLE_WAVE];
  const int rep = blockIdx.x;
  const float *lg = logits + rep * logits_rs;
  const int32_t *lab = labels + (long long)rep * B;
  T *d = dl + rep * dl_rs;
  const float invB = 1.0f / (float)B;
  float loss = 0.f;
  for (int b = threadIdx.x; b < B; b += kThreads) {
    const float *row = lg + (long long)b * C;
    float mx = row[0];
    for (int c = 1; c < C; ++c) mx = fmaxf(mx, row[c]);
    float se = 0.f;
    for (int c = 0; c < C; ++c) se += expf(row[c] - mx);
    const float lse = logf(se) + mx;
    const int y = lab[b];
    loss += lse - row[y];
    for (int c = 0; c < C; ++c) {
      const float p = expf(row[c] - lse);
      stf<T>(d, (long long)b * C + c, (p - (c == y ? 1.f : 0.f)) * invB);
    }
  }
  loss = wave_sum(loss);
  if ((threadIdx.x & (PARLE_WAVE - 1)) == 0) red[threadIdx.x / PARLE_WAVE] = loss;
  __syncthreads();
  if (threadIdx.x == 0 && loss_out) {
    float s = 0.f;
    for (int w = 0; w < kThreads / PARLE_WAVE; ++w) s += red[w];
    loss_out[rep] = s * invB;
  }
}

// ------------------------------------------------------------------ classifier head
// The last fully connected layer, the loss and that layer's input gradient in one launch: three dependent
// launches on the critical chain become one (a step of the small networks is a chain of launches of a few
// microseconds each).  One wavefront per image: lanes stride over the D features, the C <= kHeadClasses logits
// are wavefront sums (xor tree: every lane ends up with all of them), softmax and cross-entropy in registers with
// the formulas of k_softmax_train, dlogits rounded to the activation type as stored, then
//   dfeat[d] = sum_c dlogits[c] * W[c][d]   (zero where MASK and feat[d] <= 0: the ReLU in front of the layer).
// The per-image losses go to loss_img; k_loss_mean averages them (off the chain).
constexpr int kHeadClasses = 16;
constexpr int kHeadThreads = 512;  // eight wavefronts = eight images share one copy of the weights in LDS

template <typename T>
__device__ __forceinline__ float as_stored(float v);  // v after a round trip through the activation type
template <>
__device__ __forceinline__ float as_stored<float>(float v) {
  return v;
}
template <>
__device__ __forceinline__ float as_stored<bf16_t>(float v) {
  return bf16_to_f32(f32_to_bf16(v));
}

// Wavefront sums of kHeadClasses values at once, every lane receiving all of them (xor tree).  The steps of the
// tree are the outer loop: the shuffles of a step are independent and go out back to back, where one tree after
// the other would wait for every single shuffle (six dependent ones per value).
__device__ __forceinline__ void wave_allsum(float (&v)[kHeadClasses], int count) {
#pragma unroll
  for (int off = PARLE_WAVE / 2; off > 0; off >>= 1) {
    float t[kHeadClasses];
#pragma unroll
    for (int c = 0; c < kHeadClasses; ++c)
      if (c < count) t[c] = __shfl_xor(v[c], off, PARLE_WAVE);
#pragma unroll
    for (int c = 0; c < kHeadClasses; ++c)
      if (c < count) v[c] += t[c];
  }
}

template <typename T, bool MASK>
__global__ __launch_bounds__(kHeadThreads) void k_fc_head(int B, int D, int C, const T *__restrict__ feat, long long feat_rs,
                                                      const T *__restrict__ w, long long w_rs,
                                                      const float *__restrict__ bias, long long bias_rs,
                                                      const int32_t *__restrict__ labels, float *__restrict__ loss_img,
                                                      T *__restrict__ dl, long long dl_rs, T *__restrict__ dfeat,
                                                      long long dfeat_rs) {
  // the weights (shared by the workgroup's eight images) and the eight feature rows, as fp32, in LDS: both loops over
  // the features then run at LDS latency, and the weights are fetched once per workgroup
  extern __shared__ float head_lds[];
  constexpr int kWaves = kHeadThreads / PARLE_WAVE;
  float *Ws = head_lds;                 // [C][D]
  float *Fs = head_lds + (size_t)C * D;  // [kWaves][D]
  const int rep = blockIdx.y, lane = threadIdx.x & (PARLE_WAVE - 1), wave = threadIdx.x / PARLE_WAVE;
  const int b0 = blockIdx.x * kWaves, b = b0 + wave;
  const T *wp = w + rep * w_rs;
  // the image's label and the biases travel while the operands are staged
  const int y = b < B ? labels[(long long)rep * B + b] : 0;
  float bv[kHeadClasses];
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c) bv[c] = (bias && c < C) ? bias[rep * bias_rs + c] : 0.f;
  // sixteen loads in flight per thread: a loop that stores each value before it asks for the next would pay one
  // round trip to L2 per element
  auto stage = [&](float *dst, const T *src, int count) {
    constexpr int U = 16;
    for (int base = threadIdx.x; base < count; base += U * kHeadThreads) {
      float v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) v[u] = base + u * kHeadThreads < count ? ldf<T>(src, base + u * kHeadThreads) : 0.f;
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (base + u * kHeadThreads < count) dst[base + u * kHeadThreads] = v[u];
    }
  };
  stage(Ws, wp, C * D);
  stage(Fs, feat + rep * feat_rs + (long long)b0 * D, min(kWaves, B - b0) * D);
  __syncthreads();
  if (b >= B) return;  // whole wavefronts leave; no barrier follows
  const float *fs = Fs + wave * D;
  float lg[kHeadClasses];
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c) lg[c] = 0.f;
  for (int d = lane; d < D; d += PARLE_WAVE) {
    const float fv = fs[d];
#pragma unroll
    for (int c = 0; c < kHeadClasses; ++c)
      if (c < C) lg[c] += fv * Ws[c * D + d];
  }
  wave_allsum(lg, C);
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c)
    if (c < C) lg[c] += bv[c];
  float mx = lg[0];
#pragma unroll
  for (int c = 1; c < kHeadClasses; ++c)
    if (c < C) mx = fmaxf(mx, lg[c]);
  float se = 0.f;
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c)
    if (c < C) se += expf(lg[c] - mx);
  const float lse = logf(se) + mx;
  const float invB = 1.0f / (float)B;
  float ly = 0.f, mine = 0.f;
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c) {
    if (c < C) {
      if (c == y) ly = lg[c];
      const float p = expf(lg[c] - lse);
      // the gradient as the weight- and bias-gradient kernels will read it: rounded to the stored type
      lg[c] = as_stored<T>((p - (c == y ? 1.f : 0.f)) * invB);
      if (c == lane) mine = lg[c];
    }
  }
  if (lane < C) stf<T>(dl + rep * dl_rs, (long long)b * C + lane, mine);
  if (lane == 0) loss_img[(long long)rep * B + b] = lse - ly;
  T *df = dfeat + rep * dfeat_rs + (long long)b * D;
  for (int d = lane; d < D; d += PARLE_WAVE) {
    float a = 0.f;
#pragma unroll
    for (int c = 0; c < kHeadClasses; ++c)
      if (c < C) a += lg[c] * Ws[c * D + d];
    if (MASK && !(fs[d] > 0.f)) a = 0.f;
    stf<T>(df, d, a);
  }
}

// The same for a network that ends in a global average pool over class maps (All-CNN-C): logits = mean over the
// HW pixels of feat [B][HW][C], the loss, and dfeat[p][c] = dlogits[c] / HW for every pixel - pooling, loss and the
// pooling's backward pass in one launch.  One wavefront per image, lanes stride over the pixels.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_gap_head(int B, int HW, int C, const T *__restrict__ feat,
                                                       long long feat_rs, const int32_t *__restrict__ labels,
                                                       float *__restrict__ loss_img, T *__restrict__ dl, long long dl_rs,
                                                       T *__restrict__ dfeat, long long dfeat_rs) {
  const int rep = blockIdx.y, lane = threadIdx.x & (PARLE_WAVE - 1);
  const int b = blockIdx.x * (kThreads / PARLE_WAVE) + threadIdx.x / PARLE_WAVE;
  if (b >= B) return;  // whole wavefronts leave; the kernel has no barrier
  const T *f = feat + rep * feat_rs + (long long)b * HW * C;
  float lg[kHeadClasses];
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c) lg[c] = 0.f;
  for (int p = lane; p < HW; p += PARLE_WAVE) {
#pragma unroll
    for (int c = 0; c < kHeadClasses; ++c)
      if (c < C) lg[c] += ldf<T>(f, (long long)p * C + c);
  }
  const float inv = 1.0f / (float)HW;
  wave_allsum(lg, C);
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c)
    if (c < C) lg[c] *= inv;
  float mx = lg[0];
#pragma unroll
  for (int c = 1; c < kHeadClasses; ++c)
    if (c < C) mx = fmaxf(mx, lg[c]);
  float se = 0.f;
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c)
    if (c < C) se += expf(lg[c] - mx);
  const float lse = logf(se) + mx;
  const int y = labels[(long long)rep * B + b];
  const float invB = 1.0f / (float)B;
  float ly = 0.f, mine = 0.f;
#pragma unroll
  for (int c = 0; c < kHeadClasses; ++c) {
    if (c < C) {
      if (c == y) ly = lg[c];
      const float p = expf(lg[c] - lse);
      lg[c] = as_stored<T>((p - (c == y ? 1.f : 0.f)) * invB);  // dlogits as stored
      if (c == lane) mine = lg[c];
      lg[c] *= inv;                                              // the share of one pixel
    }
  }
  if (lane < C) stf<T>(dl + rep * dl_rs, (long long)b * C + lane, mine);
  if (lane == 0) loss_img[(long long)rep * B + b] = lse - ly;
  T *df = dfeat + rep * dfeat_rs + (long long)b * HW * C;
  for (int p = lane; p < HW; p += PARLE_WAVE) {
#pragma unroll
    for (int c = 0; c < kHeadClasses; ++c)
      if (c < C) stf<T>(df, (long long)p * C + c, lg[c]);
  }
}

__global__ __launch_bounds__(kThreads) void k_loss_mean(int B, const float *__restrict__ loss_img,
                                                        float *__restrict__ loss_out) {
  __shared__ float red[kThreads / PARLE_WAVE];
  const int rep = blockIdx.x;
  float s = 0.f;
  for (int b = threadIdx.x; b < B; b += kThreads) s += loss_img[(long long)rep * B + b];
  s = wave_sum(s);
  if ((threadIdx.x & (PARLE_WAVE - 1)) == 0) red[threadIdx.x / PARLE_WAVE] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < kThreads / PARLE_WAVE; ++w) t += red[w];
    loss_out[rep] = t / (float)B;
  }
}

__global__ __launch_bounds__(kThreads) void k_softmax_eval(int count, int C, const float *__restrict__ logits,
                                                           const int32_t *__restrict__ labels,
                                                           float *__restrict__ loss_sum, int32_t *__restrict__ n_err) {
  __shared__ double red[kThreads / PARLE_WAVE];
  __shared__ int redi[kThreads / PARLE_WAVE];
  double loss = 0.0;
  int err = 0;
  for (int b = threadIdx.x; b < count; b += kThreads) {
    const float *row = logits + (long long)b * C;
    float mx = row[0];
    int arg = 0;
    for (int c = 1; c < C; ++c)
      if (row[c] > mx) mx = row[c], arg = c;
    float se = 0.f;
    for (int c = 0; c < C; ++c) se += expf(row[c] - mx);
    const int y = labels[b];
    loss += (double)(logf(se) + mx - row[y]);
    err += arg != y;
  }
  loss = wave_sum(loss);
  for (int off = PARLE_WAVE / 2; off > 0; off >>= 1) err += __shfl_down(err, off, PARLE_WAVE);
  if ((threadIdx.x & (PARLE_WAVE - 1)) == 0) red[threadIdx.x / PARLE_WAVE] = loss, redi[threadIdx.x / PARLE_WAVE] = err;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    int e = 0;
    for (int w = 0; w < kThreads / PARLE_WAVE; ++w) s += red[w], e += redi[w];
    loss_sum[0] = (float)s;
    n_err[0] = e;
  }
}

// ------------------------------------------------------------------ pooling
template <typename T>
__global__ __launch_bounds__(kThreads) void k_maxpool_fwd(int B, int H, int W, int C, const T *__restrict__ in,
                                                          long long in_rs, T *__restrict__ out, long long out_rs) {
  const int Ho = H / 2, Wo = W / 2;
  const long long total = (long long)B * Ho * Wo * C;
  const T *x = in + blockIdx.y * in_rs;
  T *o = out + blockIdx.y * out_rs;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int c = i % C;
    long long t = i / C;
    const int wo = t % Wo;
    t /= Wo;
    const int ho = t % Ho;
    const int b = t / Ho;
    const long long base = (((long long)b * H + 2 * ho) * W + 2 * wo) * C + c;
    float m = ldf<T>(x, base);
    m = fmaxf(m, ldf<T>(x, base + C));
    m = fmaxf(m, ldf<T>(x, base + (long long)W * C));
    m = fmaxf(m, ldf<T>(x, base + (long long)W * C + C));
    stf<T>(o, i, m);
  }
}

// One thread per pooled element: it reads its 2 x 2 window once, finds the first maximum (row-major window
// order, as the forward pass) and writes all four input gradients; the last row / column of an odd-sized
// image belongs to no window and gets zeros from the threads of the neighbouring windows.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_maxpool_bwd(int B, int H, int W, int C, const T *__restrict__ in,
                                                          long long in_rs, const T *__restrict__ dout,
                                                          long long dout_rs, T *__restrict__ din, long long din_rs,
                                                          int relu_mask) {
  const int Ho = H / 2, Wo = W / 2;
  const long long total = (long long)B * Ho * Wo * C;
  const T *x = in + blockIdx.y * in_rs;
  const T *dy = dout + blockIdx.y * dout_rs;
  T *dx = din + blockIdx.y * din_rs;
  const long long rowC = (long long)W * C;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int c = (int)(i % C);
    long long t = i / C;
    const int wo = (int)(t % Wo);
    t /= Wo;
    const int ho = (int)(t % Ho), b = (int)(t / Ho);
    const long long base = (((long long)b * H + 2 * ho) * W + 2 * wo) * C + c;
    const float v0 = ldf<T>(x, base), v1 = ldf<T>(x, base + C), v2 = ldf<T>(x, base + rowC), v3 = ldf<T>(x, base + rowC + C);
    int arg = 0;
    float m = v0;
    if (v1 > m) m = v1, arg = 1;
    if (v2 > m) m = v2, arg = 2;
    if (v3 > m) m = v3, arg = 3;
    const float g = (!relu_mask || m > 0.f) ? ldf<T>(dy, i) : 0.f;
    stf<T>(dx, base, arg == 0 ? g : 0.f);
    stf<T>(dx, base + C, arg == 1 ? g : 0.f);
    stf<T>(dx, base + rowC, arg == 2 ? g : 0.f);
    stf<T>(dx, base + rowC + C, arg == 3 ? g : 0.f);
    const bool last_w = (W & 1) && wo == Wo - 1, last_h = (H & 1) && ho == Ho - 1;
    if (last_w) stf<T>(dx, base + 2 * C, 0.f), stf<T>(dx, base + rowC + 2 * C, 0.f);
    if (last_h) stf<T>(dx, base + 2 * rowC, 0.f), stf<T>(dx, base + 2 * rowC + C, 0.f);
    if (last_w && last_h) stf<T>(dx, base + 2 * rowC + 2 * C, 0.f);
  }
}

template <typename T, bool OUT_F32>
__global__ __launch_bounds__(kThreads) void k_gap_fwd(int B, int HW, int C, const T *__restrict__ in, long long in_rs,
                                                      void *__restrict__ out, long long out_rs) {
  const long long total = (long long)B * C;
  const T *x = in + blockIdx.y * in_rs;
  const float inv = 1.0f / (float)HW;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int c = i % C;
    const long long b = i / C;
    float s = 0.f;
    for (int p = 0; p < HW; ++p) s += ldf<T>(x, (b * HW + p) * C + c);
    if (OUT_F32)
      ((float *)out)[blockIdx.y * out_rs + i] = s * inv;
    else
      stf<T>((T *)out + blockIdx.y * out_rs, i, s * inv);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_gap_bwd(int B, int HW, int C, const T *__restrict__ dout,
                                                      long long dout_rs, T *__restrict__ din, long long din_rs) {
  const long long total = (long long)B * HW * C;
  const T *dy = dout + blockIdx.y * dout_rs;
  T *dx = din + blockIdx.y * din_rs;
  const float inv = 1.0f / (float)HW;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int c = i % C;
    const long long b = i / ((long long)HW * C);
    stf<T>(dx, i, ldf<T>(dy, b * C + c) * inv);
  }
}

// ------------------------------------------------------------------ column reductions over rows
// MODE 0: s1 = sum x.  MODE 1: s1 = sum x, s2 = sum x^2.
// MODE 2: BN-ReLU backward sums: xhat = (x - mean) rstd, pre = xhat gamma + beta, d = pre > 0 ? dy : 0;
//         s1 = sum d, s2 = sum d * xhat.
// partial layout: [rep][split][2][C] doubles.  ct = channel lanes (power of two <= 64).
template <typename T, int MODE>
__global__ __launch_bounds__(kThreads) void k_colreduce(int M, int C, int chunk, int ct, const T *__restrict__ x,
                                                        long long x_rs, const T *__restrict__ dy, long long dy_rs,
                                                        const float *__restrict__ saved, const float *__restrict__ gamma,
                                                        const float *__restrict__ beta, long long p_rs,
                                                        double *__restrict__ partial) {
  __shared__ float red[2][kThreads];
  const int rep = blockIdx.y, split = blockIdx.x, S = gridDim.x;
  const int tr = kThreads / ct;
  const int lc = threadIdx.x % ct, lr = threadIdx.x / ct;
  const int r0 = split * chunk, r1 = min(M, r0 + chunk);
  const T *xp = x + rep * x_rs;
  const T *dp = MODE == 2 ? dy + rep * dy_rs : nullptr;
  double *out = partial + ((long long)rep * S + split) * 2 * C;
  for (int cb = 0; cb < C; cb += ct) {
    const int c = cb + lc;
    float s1 = 0.f, s2 = 0.f;
    if (c < C) {
      float mean = 0.f, rstd = 0.f, gm = 0.f, bt = 0.f;
      if (MODE == 2) {
        mean = saved[(long long)rep * 2 * C + c];
        rstd = saved[(long long)rep * 2 * C + C + c];
        gm = gamma[rep * p_rs + c];
        bt = beta[rep * p_rs + c];
      }
      for (int r = r0 + lr; r < r1; r += tr) {
        const float v = ldf<T>(xp, (long long)r * C + c);
        if (MODE == 0) {
          s1 += v;
        } else if (MODE == 1) {
          s1 += v;
          s2 += v * v;
        } else {
          const float xh = (v - mean) * rstd;
          const float d = (xh * gm + bt) > 0.f ? ldf<T>(dp, (long long)r * C + c) : 0.f;
          s1 += d;
          s2 += d * xh;
        }
      }
    }
    red[0][threadIdx.x] = s1;
    red[1][threadIdx.x] = s2;
    __syncthreads();
    if (lr == 0 && c < C) {
      double a1 = 0.0, a2 = 0.0;
      for (int j = 0; j < tr; ++j) a1 += (double)red[0][j * ct + lc], a2 += (double)red[1][j * ct + lc];
      out[c] = a1;
      out[C + c] = a2;
    }
    __syncthreads();
  }
}

// Same reductions with 16-byte loads: a thread owns VW = 16/sizeof(T) consecutive channels of the
// rows r0 + lr, r0 + lr + tr, ...; row-lanes are then summed through LDS in a fixed order.
// Requires C % VW == 0 and C / VW <= 256.
template <typename T, int MODE>
__global__ __launch_bounds__(kThreads) void k_colreduce_vec(int M, int C, int chunk, const T *__restrict__ x,
                                                            long long x_rs, const T *__restrict__ dy, long long dy_rs,
                                                            const float *__restrict__ saved,
                                                            const float *__restrict__ gamma,
                                                            const float *__restrict__ beta, long long p_rs,
                                                            double *__restrict__ partial) {
  constexpr int VW = 16 / sizeof(T);
  typedef unsigned int u4v __attribute__((ext_vector_type(4)));
  __shared__ float red[2 * VW][kThreads];
  const int rep = blockIdx.y, split = blockIdx.x, S = gridDim.x;
  const int CV = C / VW, tr = kThreads / CV;
  const int lc = threadIdx.x % CV, lr = threadIdx.x / CV;
  const bool active = lr < tr;
  const int r0 = split * chunk, r1 = min(M, r0 + chunk);
  const T *xp = x + rep * x_rs;
  const T *dp = MODE == 2 ? dy + rep * dy_rs : nullptr;
  float s1[VW], s2[VW], mean[VW], rstd[VW], gm[VW], bt[VW];
#pragma unroll
  for (int e = 0; e < VW; ++e) {
    s1[e] = 0.f, s2[e] = 0.f;
    if (MODE == 2 && active) {
      const int c = lc * VW + e;
      mean[e] = saved[(long long)rep * 2 * C + c];
      rstd[e] = saved[(long long)rep * 2 * C + C + c];
      gm[e] = gamma[rep * p_rs + c];
      bt[e] = beta[rep * p_rs + c];
    }
  }
  auto unpack = [](const u4v &v, float (&f)[VW]) {
    if (sizeof(T) == 4) {
      f[0] = __uint_as_float(v.x), f[1] = __uint_as_float(v.y), f[2] = __uint_as_float(v.z), f[3] = __uint_as_float(v.w);
    } else {
      const unsigned int w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f[(2 * e) % VW] = __uint_as_float(w[e] << 16);
        f[(2 * e + 1) % VW] = __uint_as_float(w[e] & 0xffff0000u);
      }
    }
  };
  auto add_row = [&](const u4v &xq, const u4v &dq) {
    float xv[VW];
    unpack(xq, xv);
    if (MODE == 0) {
#pragma unroll
      for (int e = 0; e < VW; ++e) s1[e] += xv[e];
    } else if (MODE == 1) {
#pragma unroll
      for (int e = 0; e < VW; ++e) s1[e] += xv[e], s2[e] += xv[e] * xv[e];
    } else {
      float dv[VW];
      unpack(dq, dv);
#pragma unroll
      for (int e = 0; e < VW; ++e) {
        const float xh = (xv[e] - mean[e]) * rstd[e];
        const float d = (xh * gm[e] + bt[e]) > 0.f ? dv[e] : 0.f;
        s1[e] += d;
        s2[e] += d * xh;
      }
    }
  };
  if (active) {
    // U rows per trip, their loads issued together: a thread's trips are few (tens of rows), and with one load
    // in flight per thread the pass runs at the latency of memory, not at its bandwidth
    constexpr int U = 4;
    int r = r0 + lr;
    for (; r + (U - 1) * tr < r1; r += U * tr) {
      u4v xq[U], dq[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        xq[u] = *(const u4v *)(xp + (long long)(r + u * tr) * C + lc * VW);
        if (MODE == 2) dq[u] = *(const u4v *)(dp + (long long)(r + u * tr) * C + lc * VW);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) add_row(xq[u], dq[u]);
    }
    for (; r < r1; r += tr) {
      u4v dq = {0u, 0u, 0u, 0u};
      if (MODE == 2) dq = *(const u4v *)(dp + (long long)r * C + lc * VW);
      add_row(*(const u4v *)(xp + (long long)r * C + lc * VW), dq);
    }
  }
#pragma unroll
  for (int e = 0; e < VW; ++e) {
    red[e][threadIdx.x] = s1[e];
    red[VW + e][threadIdx.x] = s2[e];
  }
  __syncthreads();
  double *out = partial + ((long long)rep * S + split) * 2 * C;
  for (int o = threadIdx.x; o < 2 * C; o += kThreads) {
    const int k = o / C, c = o % C;
    const int slot = k * VW + c % VW, col = c / VW;
    double a = 0.0;
    for (int j = 0; j < tr; ++j) a += (double)red[slot][j * CV + col];
    out[o] = a;
  }
}

// Sum over the row-splits of one channel's two partial sums: one workgroup of kFinThreads per (channel,
// replica).  These kernels sit between two passes over the activations and last as long as their chain of
// dependent L2 round trips, so a thread takes splits t, t + kFinThreads, ... four at a time with all eight
// loads issued together (one round trip for up to 1024 splits); then a fixed shuffle tree and the wavefronts'
// sums in order (deterministic).  Every thread returns the totals.
constexpr int kFinThreads = 256;
__device__ __forceinline__ void sum_splits(const double *__restrict__ partial, int rep, int S, int C, int c, double &s1,
                                           double &s2) {
  __shared__ double red[2][kFinThreads / PARLE_WAVE];
  const double *p = partial + (long long)rep * S * 2 * C + c;
  double a1 = 0.0, a2 = 0.0;
  for (int s0 = threadIdx.x; s0 < S; s0 += 4 * kFinThreads) {
    double v1[4], v2[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int sp = s0 + u * kFinThreads;
      const bool ok = sp < S;
      v1[u] = ok ? p[(long long)sp * 2 * C] : 0.0;
      v2[u] = ok ? p[(long long)sp * 2 * C + C] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) a1 += v1[u], a2 += v2[u];
  }
  a1 = wave_sum(a1);
  a2 = wave_sum(a2);
  if ((threadIdx.x & (PARLE_WAVE - 1)) == 0) red[0][threadIdx.x / PARLE_WAVE] = a1, red[1][threadIdx.x / PARLE_WAVE] = a2;
  __syncthreads();
  s1 = 0.0, s2 = 0.0;
#pragma unroll
  for (int w = 0; w < kFinThreads / PARLE_WAVE; ++w) s1 += red[0][w], s2 += red[1][w];
}

// Bias gradient of a layer with few rows (a fully connected layer: one row per image), in one launch: a workgroup
// owns 64 channels, its four wavefronts a quarter of the rows each (row r goes to wavefront r % 4; eight loads in
// flight per thread, lanes on consecutive channels so every row is read in whole lines); the four partial sums
// are added in wavefront order.  The two-kernel reduction below would launch one workgroup per channel and
// replica to add two or three partial sums.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_bias_rows(int M, int C, const T *__restrict__ dy, long long dy_rs,
                                                        float *__restrict__ grad, long long grad_rs) {
  __shared__ double part[kThreads / PARLE_WAVE][PARLE_WAVE];
  constexpr int RL = kThreads / PARLE_WAVE;
  const int rep = blockIdx.y, lane = threadIdx.x & (PARLE_WAVE - 1), rl = threadIdx.x / PARLE_WAVE;
  const int c = blockIdx.x * PARLE_WAVE + lane;
  const T *p = dy + rep * dy_rs + (c < C ? c : 0);
  double s = 0.0;
  constexpr int U = 8;
  int r = rl;
  for (; r + (U - 1) * RL < M; r += U * RL) {
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = ldf<T>(p, (long long)(r + u * RL) * C);
#pragma unroll
    for (int u = 0; u < U; ++u) s += (double)v[u];
  }
  for (; r < M; r += RL) s += (double)ldf<T>(p, (long long)r * C);
  part[rl][lane] = s;
  __syncthreads();
  if (rl == 0 && c < C) {
    double t = part[0][lane];
#pragma unroll
    for (int w = 1; w < RL; ++w) t += part[w][lane];
    grad[rep * grad_rs + c] = (float)t;
  }
}

// bias gradient: grad[c] = sum over splits of s1
__global__ __launch_bounds__(kFinThreads) void k_bias_finalize(int C, int S, const double *__restrict__ partial,
                                                              float *__restrict__ grad, long long grad_rs) {
  const int rep = blockIdx.y, c = blockIdx.x;
  double s1, s2;
  sum_splits(partial, rep, S, C, c, s1, s2);
  if (threadIdx.x == 0) grad[rep * grad_rs + c] = (float)s1;
}

__global__ __launch_bounds__(kFinThreads) void k_bn_stats_finalize(int M, int C, int S,
                                                                  const double *__restrict__ partial,
                                                                  float *__restrict__ saved, float *__restrict__ running,
                                                                  long long run_rs) {
  const int rep = blockIdx.y, c = blockIdx.x;
  // the running statistics are fetched beside the partial sums, not in a round trip of their own after them
  float *rm = running ? running + rep * run_rs : nullptr, *rv = running ? rm + C : nullptr;
  float rm_old = 0.f, rv_old = 0.f;
  if (running && threadIdx.x == 0) rm_old = rm[c], rv_old = rv[c];
  double s1, s2;
  sum_splits(partial, rep, S, C, c, s1, s2);
  if (threadIdx.x != 0) return;
  const double mean = s1 / M;
  double var = s2 / M - mean * mean;
  if (var < 0.0) var = 0.0;
  saved[(long long)rep * 2 * C + c] = (float)mean;
  saved[(long long)rep * 2 * C + C + c] = (float)(1.0 / sqrt(var + (double)kBnEps));
  if (running) {
    const double unbiased = M > 1 ? var * ((double)M / (M - 1)) : var;
    rm[c] = (1.f - kBnMomentum) * rm_old + kBnMomentum * (float)mean;
    rv[c] = (1.f - kBnMomentum) * rv_old + kBnMomentum * (float)unbiased;
  }
}

__global__ __launch_bounds__(kThreads) void k_bn_eval_prepare(int C, const float *__restrict__ running_row,
                                                              float *__restrict__ saved) {
  const int c = blockIdx.x * kThreads + threadIdx.x;
  if (c >= C) return;
  saved[c] = running_row[c];
  saved[C + c] = 1.0f / sqrtf(running_row[C + c] + kBnEps);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_bn_apply_relu(int M, int C, const T *__restrict__ x, long long x_rs,
                                                            const float *__restrict__ gamma,
                                                            const float *__restrict__ beta, long long p_rs,
                                                            const float *__restrict__ saved, T *__restrict__ out,
                                                            long long out_rs) {
  const int rep = blockIdx.y;
  const long long total = (long long)M * C;
  const T *xp = x + rep * x_rs;
  T *op = out + rep * out_rs;
  const float *mean = saved + (long long)rep * 2 * C, *rstd = mean + C;
  const float *gm = gamma + rep * p_rs, *bt = beta + rep * p_rs;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int c = i % C;
    const float v = (ldf<T>(xp, i) - mean[c]) * rstd[c] * gm[c] + bt[c];
    stf<T>(op, i, v > 0.f ? v : 0.f);
  }
}

// 16-byte vector forms of the two BN element-wise passes (C a multiple of the vector width).
typedef unsigned int u4e __attribute__((ext_vector_type(4)));
template <typename T>
__device__ __forceinline__ void unpack16(const u4e &v, float *f) {
  if (sizeof(T) == 4) {
    f[0] = __uint_as_float(v.x), f[1] = __uint_as_float(v.y), f[2] = __uint_as_float(v.z), f[3] = __uint_as_float(v.w);
  } else {
    const unsigned int w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f[(2 * e) % (16 / sizeof(T))] = __uint_as_float(w[e] << 16);
      f[(2 * e + 1) % (16 / sizeof(T))] = __uint_as_float(w[e] & 0xffff0000u);
    }
  }
}
template <typename T>
__device__ __forceinline__ u4e pack16(const float *f) {
  u4e v;
  if (sizeof(T) == 4) {
    v.x = __float_as_uint(f[0]), v.y = __float_as_uint(f[1]), v.z = __float_as_uint(f[2]), v.w = __float_as_uint(f[3]);
  } else {
    constexpr int W = 16 / sizeof(T);
    v.x = f32x2_to_bf16x2(f[0], f[1]);
    v.y = f32x2_to_bf16x2(f[2], f[3]);
    v.z = f32x2_to_bf16x2(f[4 % W], f[5 % W]);
    v.w = f32x2_to_bf16x2(f[6 % W], f[7 % W]);
  }
  return v;
}

// bf16, C a multiple of 8: 16-byte accesses.  Forward: one workgroup per image; a thread owns 8 channels of the
// pixels pl, pl + PL, ... (PL = 256 / (C / 8) pixel lanes, several loads in flight), the lanes' sums are added
// through LDS in lane order.  Backward: one thread per 16-byte vector of the input gradient.
template <bool OUT_F32>
__global__ __launch_bounds__(kThreads) void k_gap_fwd_vec(int HW, int C, const bf16_t *__restrict__ in, long long in_rs,
                                                          void *__restrict__ out, long long out_rs) {
  __shared__ float red[kThreads * 8];
  const int b = blockIdx.x, rep = blockIdx.y;
  const int CV = C >> 3, PL = kThreads / CV;
  const int cv = threadIdx.x % CV, pl = threadIdx.x / CV;
  const bf16_t *x = in + rep * in_rs + (long long)b * HW * C + cv * 8;
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (pl < PL) {
#pragma unroll 4
    for (int p = pl; p < HW; p += PL) {
      float v[8];
      unpack16<bf16_t>(*(const u4e *)(x + (long long)p * C), v);
#pragma unroll
      for (int e = 0; e < 8; ++e) s[e] += v[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[pl * C + cv * 8 + e] = s[e];
  }
  __syncthreads();
  const float inv = 1.0f / (float)HW;
  for (int c = threadIdx.x; c < C; c += kThreads) {
    float t = 0.f;
    for (int l = 0; l < PL; ++l) t += red[l * C + c];
    const long long o = rep * out_rs + (long long)b * C + c;
    if (OUT_F32)
      ((float *)out)[o] = t * inv;
    else
      ((bf16_t *)out)[o] = f32_to_bf16(t * inv);
  }
}

__global__ __launch_bounds__(kThreads) void k_gap_bwd_vec(long long total, int HW, int CV, const bf16_t *__restrict__ dout,
                                                          long long dout_rs, bf16_t *__restrict__ din, long long din_rs) {
  const bf16_t *dy = dout + blockIdx.y * dout_rs;
  bf16_t *dx = din + blockIdx.y * din_rs;
  const float inv = 1.0f / (float)HW;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int cv = (int)(i % CV);
    const long long b = i / ((long long)HW * CV);
    float v[8];
    unpack16<bf16_t>(*(const u4e *)(dy + (b * CV + cv) * 8), v);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= inv;
    *(u4e *)(dx + i * 8) = pack16<bf16_t>(v);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_bn_apply_relu_vec(int M, int C, const T *__restrict__ x, long long x_rs,
                                                                const float *__restrict__ gamma,
                                                                const float *__restrict__ beta, long long p_rs,
                                                                const float *__restrict__ saved, T *__restrict__ out,
                                                                long long out_rs) {
  constexpr int VW = 16 / sizeof(T);
  const int rep = blockIdx.y;
  const int CV = C / VW;
  const long long total = (long long)M * CV;
  const T *xp = x + rep * x_rs;
  T *op = out + rep * out_rs;
  const float *mean = saved + (long long)rep * 2 * C, *rstd = mean + C;
  const float *gm = gamma + rep * p_rs, *bt = beta + rep * p_rs;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int c0 = (int)(i % CV) * VW;
    float xv[VW], ov[VW];
    unpack16<T>(*(const u4e *)(xp + i * VW), xv);
#pragma unroll
    for (int e = 0; e < VW; ++e) {
      const float v = (xv[e] - mean[c0 + e]) * rstd[c0 + e] * gm[c0 + e] + bt[c0 + e];
      ov[e] = v > 0.f ? v : 0.f;
    }
    *(u4e *)(op + i * VW) = pack16<T>(ov);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_bn_bwd_apply_vec(int M, int C, const T *__restrict__ x, long long x_rs,
                                                               const T *__restrict__ dout, long long dout_rs,
                                                               const float *__restrict__ gamma,
                                                               const float *__restrict__ beta, long long p_rs,
                                                               const float *__restrict__ saved,
                                                               const float *__restrict__ sums, const T *__restrict__ add,
                                                               long long add_rs, T *__restrict__ dx, long long dx_rs) {
  constexpr int VW = 16 / sizeof(T);
  const int rep = blockIdx.y;
  const int CV = C / VW;
  const long long total = (long long)M * CV;
  const T *xp = x + rep * x_rs;
  const T *dp = dout + rep * dout_rs;
  const T *ap = add ? add + rep * add_rs : nullptr;
  T *op = dx + rep * dx_rs;
  const float *mean = saved + (long long)rep * 2 * C, *rstd = mean + C;
  const float *s1 = sums + (long long)rep * 2 * C, *s2 = s1 + C;
  const float *gm = gamma + rep * p_rs, *bt = beta + rep * p_rs;
  const float invM = 1.0f / (float)M;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int c0 = (int)(i % CV) * VW;
    float xv[VW], dv[VW], av[VW], ov[VW];
    unpack16<T>(*(const u4e *)(xp + i * VW), xv);
    unpack16<T>(*(const u4e *)(dp + i * VW), dv);
    if (ap) unpack16<T>(*(const u4e *)(ap + i * VW), av);
#pragma unroll
    for (int e = 0; e < VW; ++e) {
      const int c = c0 + e;
      const float xh = (xv[e] - mean[c]) * rstd[c];
      const float d = (xh * gm[c] + bt[c]) > 0.f ? dv[e] : 0.f;
      float v = gm[c] * rstd[c] * (d - s1[c] * invM - xh * s2[c] * invM);
      if (ap) v += av[e];
      ov[e] = v;
    }
    *(u4e *)(op + i * VW) = pack16<T>(ov);
  }
}

__global__ __launch_bounds__(kFinThreads) void k_bn_bwd_finalize(int C, int S, const double *__restrict__ partial,
                                                                float *__restrict__ sums, float *__restrict__ dgamma,
                                                                float *__restrict__ dbeta, long long p_rs) {
  const int rep = blockIdx.y, c = blockIdx.x;
  double s1, s2;
  sum_splits(partial, rep, S, C, c, s1, s2);
  if (threadIdx.x != 0) return;
  sums[(long long)rep * 2 * C + c] = (float)s1;
  sums[(long long)rep * 2 * C + C + c] = (float)s2;
  dbeta[rep * p_rs + c] = (float)s1;
  dgamma[rep * p_rs + c] = (float)s2;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_bn_bwd_apply(int M, int C, const T *__restrict__ x, long long x_rs,
                                                           const T *__restrict__ dout, long long dout_rs,
                                                           const float *__restrict__ gamma,
                                                           const float *__restrict__ beta, long long p_rs,
                                                           const float *__restrict__ saved,
                                                           const float *__restrict__ sums, const T *__restrict__ add,
                                                           long long add_rs, T *__restrict__ dx, long long dx_rs) {
  const int rep = blockIdx.y;
  const long long total = (long long)M * C;
  const T *xp = x + rep * x_rs;
  const T *dp = dout + rep * dout_rs;
  const T *ap = add ? add + rep * add_rs : nullptr;
  T *op = dx + rep * dx_rs;
  const float *mean = saved + (long long)rep * 2 * C, *rstd = mean + C;
  const float *s1 = sums + (long long)rep * 2 * C, *s2 = s1 + C;
  const float *gm = gamma + rep * p_rs, *bt = beta + rep * p_rs;
  const float invM = 1.0f / (float)M;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int c = i % C;
    const float xh = (ldf<T>(xp, i) - mean[c]) * rstd[c];
    const float d = (xh * gm[c] + bt[c]) > 0.f ? ldf<T>(dp, i) : 0.f;
    float v = gm[c] * rstd[c] * (d - s1[c] * invM - xh * s2[c] * invM);
    if (ap) v += ldf<T>(ap, i);
    stf<T>(op, i, v);
  }
}

// ------------------------------------------------------------------ small utilities
__global__ __launch_bounds__(kThreads) void k_reduce_partials(int S, long long len, const float *__restrict__ partial,
                                                              float *__restrict__ out, long long out_rs) {
  const int rep = blockIdx.y;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < len; i += (long long)gridDim.x * kThreads) {
    float s = 0.f;
    for (int sp = 0; sp < S; ++sp) s += partial[((long long)rep * S + sp) * len + i];
    out[rep * out_rs + i] = s;
  }
}

// Same sum for lengths that are a multiple of four: a block owns 64 vectors of four columns, its
// four wavefronts each add a contiguous quarter of the splits (loads 16 bytes wide, eight in
// flight), and the four sums are combined in a fixed order through LDS.  The grouping depends only
// on S, so the result is reproducible run to run.
__global__ __launch_bounds__(kThreads) void k_reduce_partials_v(int S, long long len4, const f4 *__restrict__ partial,
                                                                f4 *__restrict__ out, long long out_rs4) {
  __shared__ f4 part[3][64];
  const int rep = blockIdx.y, lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const long long i = (long long)blockIdx.x * 64 + lane;
  const int per = (S + 3) / 4, sp0 = grp * per, sp1 = min(S, sp0 + per);
  f4 s = {0.f, 0.f, 0.f, 0.f};
  if (i < len4) {
    const f4 *src = partial + (long long)rep * S * len4 + i;
    int sp = sp0;
    for (; sp + 8 <= sp1; sp += 8) {
      f4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + (long long)(sp + u) * len4);
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; sp < sp1; ++sp) s += __builtin_nontemporal_load(src + (long long)sp * len4);
  }
  if (grp) part[grp - 1][lane] = s;
  __syncthreads();
  if (grp == 0 && i < len4) {
    s += part[0][lane];
    s += part[1][lane];
    s += part[2][lane];
    out[rep * out_rs4 + i] = s;
  }
}

// Few splits: one thread per vector of four columns adds all of them in order, eight loads in flight; no LDS, no
// barrier, a quarter of the workgroups.
__global__ __launch_bounds__(kThreads) void k_reduce_partials_t(int S, long long len4, const f4 *__restrict__ partial,
                                                                f4 *__restrict__ out, long long out_rs4) {
  const int rep = blockIdx.y;
  const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (i >= len4) return;
  const f4 *src = partial + (long long)rep * S * len4 + i;
  f4 s = {0.f, 0.f, 0.f, 0.f};
  int sp = 0;
  for (; sp + 8 <= S; sp += 8) {
    f4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + (long long)(sp + u) * len4);
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  for (; sp < S; ++sp) s += __builtin_nontemporal_load(src + (long long)sp * len4);
  out[rep * out_rs4 + i] = s;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_weight_transpose(int Cout, int RS, int Cin, const T *__restrict__ w,
                                                               long long w_rs, T *__restrict__ wt, long long wt_rs) {
  const long long total = (long long)Cout * RS * Cin;
  const T *src = w + blockIdx.y * w_rs;
  T *dst = wt + blockIdx.y * wt_rs;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int co = i % Cout;
    long long t = i / Cout;
    const int rs = t % RS;
    const int ci = t / RS;
    dst[i] = src[((long long)co * RS + rs) * Cin + ci];
  }
}

// For every window tap rs the layer is a [Cout][Cin] matrix (row stride RS*Cin) that becomes a
// [Cin][Cout] matrix (row stride RS*Cout): 64 x 64 tiles go through LDS so that both the reads (along
// Cin) and the writes (along Cout) are contiguous.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_weight_transpose_all(const TransposeTable tab, const T *__restrict__ params,
                                                                   long long p_rs, char *__restrict__ dst_base) {
  __shared__ T tile[64][64 + 2];
  const int layer = blockIdx.y, rep = blockIdx.z;
  const int Cout = tab.cout[layer], RS = tab.rs[layer], Cin = tab.cin[layer];
  const long long total = (long long)Cout * RS * Cin;
  const T *src = params + rep * p_rs + tab.src_off[layer];
  T *dst = (T *)(dst_base + tab.dst_off[layer]) + (long long)rep * total;
  const int tco = (Cout + 63) / 64, tci = (Cin + 63) / 64;
  const int tiles = tco * tci * RS;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 x 4
  for (int t = blockIdx.x; t < tiles; t += gridDim.x) {
    const int rs = t % RS, tt = t / RS;
    const int co0 = (tt / tci) * 64, ci0 = (tt % tci) * 64;
#pragma unroll 4
    for (int r = ty; r < 64; r += 4) {
      const int co = co0 + r, ci = ci0 + tx;
      if (co < Cout && ci < Cin) tile[r][tx] = src[((long long)co * RS + rs) * Cin + ci];
    }
    __syncthreads();
#pragma unroll 4
    for (int r = ty; r < 64; r += 4) {
      const int ci = ci0 + r, co = co0 + tx;
      if (ci < Cin && co < Cout)
        dst[(tab.tap_major[layer] ? (long long)rs * Cin + ci : (long long)ci * RS + rs) * Cout + co] = tile[tx][r];
    }
    __syncthreads();
  }
}

// Second half of a backward-data pass that goes through per-tap products: col[m][(r*S + s)*Cin + ci] holds
// dy[m] . w[:, r, s, ci] for every output pixel m = (b, p, q) (a plain matrix product over the output
// channels); the input gradient of pixel (h, w) is the sum of the entries whose window covers it,
//   dx[b, h, w, ci] = sum_{r, s} col[(b, h + pad - r, w + pad - s)][(r*S + s)*Cin + ci]   (stride 1),
// taken in tap order.  One thread per (pixel, channel): neighbouring threads read neighbouring channels of
// one tap; a row of col is read by the R*S pixels around it.
__global__ __launch_bounds__(kThreads) void k_col2im(int B, int H, int W, int Cin, int R, int pad, int P, int Q,
                                                     const float *__restrict__ col, long long col_rs,
                                                     const float *__restrict__ mask, long long mask_rs, int accumulate,
                                                     float *__restrict__ dx, long long dx_rs) {
  const int rep = blockIdx.y;
  const long long total = (long long)B * H * W * Cin;
  const int RS = R * R, ldc = Cin * RS;
  const float *cp = col + rep * col_rs;
  const float *mp = mask ? mask + rep * mask_rs : nullptr;
  float *op = dx + rep * dx_rs;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < total; i += (long long)gridDim.x * kThreads) {
    const int ci = (int)(i % Cin);
    long long pix = i / Cin;
    const int w = (int)(pix % W);
    pix /= W;
    const int h = (int)(pix % H), b = (int)(pix / H);
    float sum = 0.f;
    for (int r = 0; r < R; ++r) {
      const int p = h + pad - r;
      if (p < 0 || p >= P) continue;
      for (int s2 = 0; s2 < R; ++s2) {
        const int q = w + pad - s2;
        if (q < 0 || q >= Q) continue;
        sum += cp[((long long)(b * P + p) * Q + q) * ldc + (r * R + s2) * Cin + ci];
      }
    }
    if (mp && !(mp[i] > 0.f)) sum = 0.f;
    op[i] = accumulate ? op[i] + sum : sum;
  }
}

// Same transposition for layers whose channel counts fill whole 16-byte vectors: one workgroup per tile (found
// by a scan of the table's running tile counts), 16-byte loads along Cin and 16-byte stores along Cout; only
// the column reads from LDS are element-wise.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_weight_transpose_vec(const TransposeTable tab, const T *__restrict__ params,
                                                                   long long p_rs, char *__restrict__ dst_base) {
  constexpr int VW = 16 / sizeof(T), VPR = 64 / VW;  // vectors per tile row
  __shared__ __attribute__((aligned(16))) T tile[64][64 + VW];
  int layer = 0;
  while (layer + 1 < tab.count && (int)blockIdx.x >= tab.tile_begin[layer + 1]) ++layer;
  const int rep = blockIdx.y;
  const int Cout = tab.cout[layer], RS = tab.rs[layer], Cin = tab.cin[layer];
  const long long total = (long long)Cout * RS * Cin;
  const T *src = params + rep * p_rs + tab.src_off[layer];
  T *dst = (T *)(dst_base + tab.dst_off[layer]) + (long long)rep * total;
  const int tci = (Cin + 63) / 64;
  const int t = blockIdx.x - tab.tile_begin[layer];
  const int rs = t % RS, tt = t / RS;
  const int co0 = (tt / tci) * 64, ci0 = (tt % tci) * 64;
#pragma unroll
  for (int v = threadIdx.x; v < 64 * VPR; v += kThreads) {
    const int r = v / VPR, c = (v % VPR) * VW;
    const int co = co0 + r, ci = ci0 + c;
    if (co < Cout && ci < Cin) *(uint4 *)&tile[r][c] = *(const uint4 *)&src[((long long)co * RS + rs) * Cin + ci];
  }
  __syncthreads();
#pragma unroll
  for (int v = threadIdx.x; v < 64 * VPR; v += kThreads) {
    const int r = v / VPR, c = (v % VPR) * VW;  // r: input channel of the row, c: first of VW output channels
    const int ci = ci0 + r, co = co0 + c;
    if (ci < Cin && co < Cout) {
      union {
        T e[VW];
        uint4 q;
      } out;
#pragma unroll
      for (int e = 0; e < VW; ++e) out.e[e] = tile[c + e][r];
      *(uint4 *)&dst[(tab.tap_major[layer] ? (long long)rs * Cin + ci : (long long)ci * RS + rs) * Cout + co] = out.q;
    }
  }
}

__device__ __forceinline__ unsigned mix32(unsigned x) {
  x ^= x >> 16;
  x *= 0x7FEB352Du;
  x ^= x >> 15;
  x *= 0x846CA68Bu;
  x ^= x >> 16;
  return x;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_dropout(long long count, const T *__restrict__ in, long long in_rs,
                                                      T *__restrict__ out, long long out_rs,
                                                      const T *__restrict__ relu_src, long long relu_rs, unsigned seed,
                                                      const long long *__restrict__ step_dev, unsigned site,
                                                      unsigned thresh, float scale) {
  const unsigned rep = blockIdx.y;
  const unsigned k = step_dev ? (unsigned)step_dev[0] : 0u;
  unsigned key = mix32(seed + 0x9E3779B9u * k);
  key = mix32(key ^ (rep * 0x85EBCA6Bu + site * 0xC2B2AE35u + 1u));
  const T *ip = in + rep * in_rs;
  T *op = out + rep * out_rs;
  const T *rp = relu_src ? relu_src + rep * relu_rs : nullptr;
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < count; i += (long long)gridDim.x * kThreads) {
    const unsigned h = mix32(mix32((unsigned)i ^ key) + key);
    float v = (h >> 8) >= thresh ? ldf<T>(ip, i) * scale : 0.f;
    if (rp && !(ldf<T>(rp, i) > 0.f)) v = 0.f;
    stf<T>(op, i, v);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_convert(const float *__restrict__ src, T *__restrict__ dst,
                                                      long long count) {
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < count; i += (long long)gridDim.x * kThreads)
    stf<T>(dst, i, src[i]);
}

__global__ __launch_bounds__(kThreads) void k_fill(float *__restrict__ dst, long long count, float v) {
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < count; i += (long long)gridDim.x * kThreads)
    dst[i] = v;
}

__global__ __launch_bounds__(kThreads) void k_row_mean(int n, long long len, const float *__restrict__ in, long long rs,
                                                       float *__restrict__ out) {
  for (long long i = (long long)blockIdx.x * kThreads + threadIdx.x; i < len; i += (long long)gridDim.x * kThreads) {
    float s = 0.f;
    for (int a = 0; a < n; ++a) s += in[a * rs + i];
    out[i] = s / (float)n;
  }
}

template <typename T, int MODE>
void run_colreduce(hipStream_t st, dim3 grid, int M, int C, int chunk, int ct, const void *x, long long x_rs,
                   const void *dy, long long dy_rs, const float *saved, const float *gamma, const float *beta,
                   long long p_rs, double *partial) {
  constexpr int VW = 16 / sizeof(T);
  const bool vec = C % VW == 0 && C / VW <= kThreads && x_rs % VW == 0 && dy_rs % VW == 0 &&
                   (reinterpret_cast<uintptr_t>(x) & 15) == 0 && (reinterpret_cast<uintptr_t>(dy) & 15) == 0;
  if (vec)
    hipLaunchKernelGGL((k_colreduce_vec<T, MODE>), grid, dim3(kThreads), 0, st, M, C, chunk, (const T *)x, x_rs,
                       (const T *)dy, dy_rs, saved, gamma, beta, p_rs, partial);
  else
    hipLaunchKernelGGL((k_colreduce<T, MODE>), grid, dim3(kThreads), 0, st, M, C, chunk, ct, (const T *)x, x_rs,
                       (const T *)dy, dy_rs, saved, gamma, beta, p_rs, partial);
}

int channel_lanes(int C) {
  int ct = 1;
  while (ct < C && ct < 64) ct <<= 1;
  return ct;
}

int col_chunk(int M, int S) {
  int chunk = (M + S - 1) / S;
  return chunk < 1 ? 1 : chunk;
}

}  // namespace

#define DISPATCH_T(dtype, CALL_F32, CALL_BF16) \
  do {                                         \
    if ((dtype) == 0) {                        \
      CALL_F32;                                \
    } else {                                   \
      CALL_BF16;                               \
    }                                          \
  } while (0)

hipError_t launch_softmax_xent_train(hipStream_t st, int dtype, int n, int B, int C, const float *logits,
                                     long long logits_rs, const int32_t *labels, float *loss_out, void *dlogits,
                                     long long dl_rs) {
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_softmax_train<float>, dim3(n), dim3(kThreads), 0, st, B, C, logits, logits_rs, labels,
                                loss_out, (float *)dlogits, dl_rs),
             hipLaunchKernelGGL(k_softmax_train<bf16_t>, dim3(n), dim3(kThreads), 0, st, B, C, logits, logits_rs,
                                labels, loss_out, (bf16_t *)dlogits, dl_rs));
  return hipGetLastError();
}

// at most 16 classes (registers), weights and eight feature rows within 64 KB of LDS
bool fc_head_applicable(int classes, int features) {
  return classes >= 1 && classes <= kHeadClasses && features >= 1 &&
         ((long long)classes + kHeadThreads / PARLE_WAVE) * features * 4 <= 65536;
}

hipError_t launch_fc_head(hipStream_t st, int dtype, int n, int B, int D, int C, const void *feat, long long feat_rs,
                          const void *w, long long w_rs, const float *bias, long long bias_rs, const int32_t *labels,
                          float *loss_img, void *dlogits, long long dl_rs, void *dfeat, long long dfeat_rs, bool mask) {
  if (!fc_head_applicable(C, D) || B < 1) return hipErrorInvalidValue;
  const dim3 grid((B + kHeadThreads / PARLE_WAVE - 1) / (kHeadThreads / PARLE_WAVE), n);
  const size_t lds = (size_t)(C + kHeadThreads / PARLE_WAVE) * D * sizeof(float);
#define HEAD(T, MASK)                                                                                                  \
  hipLaunchKernelGGL((k_fc_head<T, MASK>), grid, dim3(kHeadThreads), lds, st, B, D, C, (const T *)feat, feat_rs, (const T *)w, \
                     w_rs, bias, bias_rs, labels, loss_img, (T *)dlogits, dl_rs, (T *)dfeat, dfeat_rs)
  if (dtype == 0) {
    if (mask) HEAD(float, true); else HEAD(float, false);
  } else {
    if (mask) HEAD(bf16_t, true); else HEAD(bf16_t, false);
  }
#undef HEAD
  return hipGetLastError();
}

hipError_t launch_gap_head(hipStream_t st, int dtype, int n, int B, int HW, int C, const void *feat, long long feat_rs,
                           const int32_t *labels, float *loss_img, void *dlogits, long long dl_rs, void *dfeat,
                           long long dfeat_rs) {
  if (C < 1 || C > kHeadClasses || B < 1 || HW < 1) return hipErrorInvalidValue;
  const dim3 grid((B + kThreads / PARLE_WAVE - 1) / (kThreads / PARLE_WAVE), n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_gap_head<float>, grid, dim3(kThreads), 0, st, B, HW, C, (const float *)feat, feat_rs,
                                labels, loss_img, (float *)dlogits, dl_rs, (float *)dfeat, dfeat_rs),
             hipLaunchKernelGGL(k_gap_head<bf16_t>, grid, dim3(kThreads), 0, st, B, HW, C, (const bf16_t *)feat, feat_rs,
                                labels, loss_img, (bf16_t *)dlogits, dl_rs, (bf16_t *)dfeat, dfeat_rs));
  return hipGetLastError();
}

hipError_t launch_loss_mean(hipStream_t st, int n, int B, const float *loss_img, float *loss_out) {
  hipLaunchKernelGGL(k_loss_mean, dim3(n), dim3(kThreads), 0, st, B, loss_img, loss_out);
  return hipGetLastError();
}

hipError_t launch_softmax_xent_eval(hipStream_t st, int count, int C, const float *logits, const int32_t *labels,
                                    float *loss_sum, int32_t *n_err) {
  hipLaunchKernelGGL(k_softmax_eval, dim3(1), dim3(kThreads), 0, st, count, C, logits, labels, loss_sum, n_err);
  return hipGetLastError();
}

hipError_t launch_maxpool_fwd(hipStream_t st, int dtype, int n, int B, int H, int W, int C, const void *in,
                              long long in_rs, void *out, long long out_rs) {
  dim3 grid(blocks_for((long long)B * (H / 2) * (W / 2) * C, 65535), n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_maxpool_fwd<float>, grid, dim3(kThreads), 0, st, B, H, W, C, (const float *)in, in_rs,
                                (float *)out, out_rs),
             hipLaunchKernelGGL(k_maxpool_fwd<bf16_t>, grid, dim3(kThreads), 0, st, B, H, W, C, (const bf16_t *)in,
                                in_rs, (bf16_t *)out, out_rs));
  return hipGetLastError();
}

hipError_t launch_maxpool_bwd(hipStream_t st, int dtype, int n, int B, int H, int W, int C, const void *in,
                              long long in_rs, const void *dout, long long dout_rs, void *din, long long din_rs,
                              int relu_mask) {
  if (H < 2 || W < 2) return hipErrorInvalidValue;  // no window: the plans never pool such a tensor
  dim3 grid(blocks_for((long long)B * (H / 2) * (W / 2) * C, 65535), n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_maxpool_bwd<float>, grid, dim3(kThreads), 0, st, B, H, W, C, (const float *)in, in_rs,
                                (const float *)dout, dout_rs, (float *)din, din_rs, relu_mask),
             hipLaunchKernelGGL(k_maxpool_bwd<bf16_t>, grid, dim3(kThreads), 0, st, B, H, W, C, (const bf16_t *)in,
                                in_rs, (const bf16_t *)dout, dout_rs, (bf16_t *)din, din_rs, relu_mask));
  return hipGetLastError();
}

hipError_t launch_col2im(hipStream_t st, int n, int B, int H, int W, int Cin, int R, int pad, const float *col,
                         long long col_rs, const float *mask, long long mask_rs, int accumulate, float *dx,
                         long long dx_rs) {
  const int P = H + 2 * pad - R + 1, Q = W + 2 * pad - R + 1;
  if (P < 1 || Q < 1) return hipErrorInvalidValue;
  dim3 grid(blocks_for((long long)B * H * W * Cin, 65535), n);
  hipLaunchKernelGGL(k_col2im, grid, dim3(kThreads), 0, st, B, H, W, Cin, R, pad, P, Q, col, col_rs, mask, mask_rs,
                     accumulate, dx, dx_rs);
  return hipGetLastError();
}

hipError_t launch_gap_fwd(hipStream_t st, int dtype, bool out_f32, int n, int B, int HW, int C, const void *in,
                          long long in_rs, void *out, long long out_rs) {
  if (dtype == 1 && C % 8 == 0 && C / 8 <= kThreads && in_rs % 8 == 0 && aligned_to(in, 16)) {
    dim3 vgrid(B, n);
    if (out_f32)
      hipLaunchKernelGGL(k_gap_fwd_vec<true>, vgrid, dim3(kThreads), 0, st, HW, C, (const bf16_t *)in, in_rs, out, out_rs);
    else
      hipLaunchKernelGGL(k_gap_fwd_vec<false>, vgrid, dim3(kThreads), 0, st, HW, C, (const bf16_t *)in, in_rs, out, out_rs);
    return hipGetLastError();
  }
  dim3 grid(blocks_for((long long)B * C, 65535), n);
  if (dtype == 0) {
    hipLaunchKernelGGL((k_gap_fwd<float, true>), grid, dim3(kThreads), 0, st, B, HW, C, (const float *)in, in_rs, out,
                       out_rs);
  } else if (out_f32) {
    hipLaunchKernelGGL((k_gap_fwd<bf16_t, true>), grid, dim3(kThreads), 0, st, B, HW, C, (const bf16_t *)in, in_rs, out,
                       out_rs);
  } else {
    hipLaunchKernelGGL((k_gap_fwd<bf16_t, false>), grid, dim3(kThreads), 0, st, B, HW, C, (const bf16_t *)in, in_rs,
                       out, out_rs);
  }
  return hipGetLastError();
}

hipError_t launch_gap_bwd(hipStream_t st, int dtype, int n, int B, int HW, int C, const void *dout, long long dout_rs,
                          void *din, long long din_rs) {
  if (dtype == 1 && C % 8 == 0 && dout_rs % 8 == 0 && din_rs % 8 == 0 && aligned_to(dout, 16) && aligned_to(din, 16)) {
    const long long total = (long long)B * HW * (C / 8);
    hipLaunchKernelGGL(k_gap_bwd_vec, dim3(blocks_for(total, 65535), n), dim3(kThreads), 0, st, total, HW, C / 8,
                       (const bf16_t *)dout, dout_rs, (bf16_t *)din, din_rs);
    return hipGetLastError();
  }
  dim3 grid(blocks_for((long long)B * HW * C, 65535), n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_gap_bwd<float>, grid, dim3(kThreads), 0, st, B, HW, C, (const float *)dout, dout_rs,
                                (float *)din, din_rs),
             hipLaunchKernelGGL(k_gap_bwd<bf16_t>, grid, dim3(kThreads), 0, st, B, HW, C, (const bf16_t *)dout, dout_rs,
                                (bf16_t *)din, din_rs));
  return hipGetLastError();
}

int colreduce_splits(int n, int M) {
  // two workgroups per compute unit (more splits cost the finalize kernel more than they gain the reduction:
  // measured 256 .. 2048), at least 64 rows per split
  int want = (512 + n - 1) / n;
  int maxs = (M + 63) / 64;
  if (want > maxs) want = maxs;
  if (want < 1) want = 1;
  if (want > 1024) want = 1024;
  return want;
}

hipError_t launch_bias_grad(hipStream_t st, int dtype, int n, int M, int C, const void *dy, long long dy_rs,
                            double *partial, float *grad, long long grad_rs) {
  if (M <= 512) {  // fully connected layers
    dim3 rgrid((C + PARLE_WAVE - 1) / PARLE_WAVE, n);
    DISPATCH_T(dtype,
               hipLaunchKernelGGL(k_bias_rows<float>, rgrid, dim3(kThreads), 0, st, M, C, (const float *)dy, dy_rs, grad,
                                  grad_rs),
               hipLaunchKernelGGL(k_bias_rows<bf16_t>, rgrid, dim3(kThreads), 0, st, M, C, (const bf16_t *)dy, dy_rs, grad,
                                  grad_rs));
    return hipGetLastError();
  }
  const int S = colreduce_splits(n, M), chunk = col_chunk(M, S), ct = channel_lanes(C);
  dim3 grid(S, n);
  DISPATCH_T(dtype,
             (run_colreduce<float, 0>(st, grid, M, C, chunk, ct, dy, dy_rs, nullptr, 0LL, nullptr, nullptr, nullptr, 0LL,
                                      partial)),
             (run_colreduce<bf16_t, 0>(st, grid, M, C, chunk, ct, dy, dy_rs, nullptr, 0LL, nullptr, nullptr, nullptr, 0LL,
                                       partial)));
  hipLaunchKernelGGL(k_bias_finalize, dim3(C, n), dim3(kFinThreads), 0, st, C, S, partial, grad, grad_rs);
  return hipGetLastError();
}

hipError_t launch_reduce_partials(hipStream_t st, int n, int S, long long len, const float *partial, float *out,
                                  long long out_rs) {
  static const int t_max = [] {
    const char *e = getenv("PARLE_REDUCE_T");  // splits up to which the one-thread-per-vector form runs
    return e ? atoi(e) : 32;
  }();
  if (len % 4 == 0 && out_rs % 4 == 0 && aligned_to(partial, 16) && aligned_to(out, 16) && S <= t_max) {
    hipLaunchKernelGGL(k_reduce_partials_t, dim3((unsigned)((len / 4 + kThreads - 1) / kThreads), n), dim3(kThreads), 0, st, S,
                       len / 4, (const f4 *)partial, (f4 *)out, out_rs / 4);
    return hipGetLastError();
  }
  if (len % 4 == 0 && out_rs % 4 == 0 && aligned_to(partial, 16) && aligned_to(out, 16) && len / 4 / 64 < (1LL << 31)) {
    hipLaunchKernelGGL(k_reduce_partials_v, dim3((unsigned)((len / 4 + 63) / 64), n), dim3(kThreads), 0, st, S, len / 4,
                       (const f4 *)partial, (f4 *)out, out_rs / 4);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(k_reduce_partials, dim3(blocks_for(len, 65535), n), dim3(kThreads), 0, st, S, len, partial, out,
                     out_rs);
  return hipGetLastError();
}

hipError_t launch_bn_train_fwd(hipStream_t st, int dtype, int n, int M, int C, const void *x, long long x_rs,
                               const float *gamma, const float *beta, long long p_rs, double *partial, int pre_splits,
                               float *saved, float *running, long long run_rs, void *out, long long out_rs) {
  // pre_splits > 0: the kernel that wrote x has left that many partial rows of column sums in `partial`
  const int S = pre_splits > 0 ? pre_splits : colreduce_splits(n, M);
  if (pre_splits <= 0) {
    const int chunk = col_chunk(M, S), ct = channel_lanes(C);
    dim3 grid(S, n);
    DISPATCH_T(dtype,
               (run_colreduce<float, 1>(st, grid, M, C, chunk, ct, x, x_rs, nullptr, 0LL, nullptr, nullptr, nullptr, 0LL,
                                        partial)),
               (run_colreduce<bf16_t, 1>(st, grid, M, C, chunk, ct, x, x_rs, nullptr, 0LL, nullptr, nullptr, nullptr,
                                         0LL, partial)));
  }
  hipLaunchKernelGGL(k_bn_stats_finalize, dim3(C, n), dim3(kFinThreads), 0, st, M, C, S, partial, saved, running,
                     run_rs);
  const int vw = dtype ? 8 : 4;
  if (C % vw == 0 && x_rs % vw == 0 && out_rs % vw == 0 && aligned_to(x, 16) && aligned_to(out, 16)) {
    dim3 vgrid(blocks_for((long long)M * (C / vw), 8192), n);
    DISPATCH_T(dtype,
               hipLaunchKernelGGL(k_bn_apply_relu_vec<float>, vgrid, dim3(kThreads), 0, st, M, C, (const float *)x, x_rs,
                                  gamma, beta, p_rs, saved, (float *)out, out_rs),
               hipLaunchKernelGGL(k_bn_apply_relu_vec<bf16_t>, vgrid, dim3(kThreads), 0, st, M, C, (const bf16_t *)x,
                                  x_rs, gamma, beta, p_rs, saved, (bf16_t *)out, out_rs));
    return hipGetLastError();
  }
  dim3 agrid(blocks_for((long long)M * C, 4096), n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_bn_apply_relu<float>, agrid, dim3(kThreads), 0, st, M, C, (const float *)x, x_rs, gamma,
                                beta, p_rs, saved, (float *)out, out_rs),
             hipLaunchKernelGGL(k_bn_apply_relu<bf16_t>, agrid, dim3(kThreads), 0, st, M, C, (const bf16_t *)x, x_rs,
                                gamma, beta, p_rs, saved, (bf16_t *)out, out_rs));
  return hipGetLastError();
}

hipError_t launch_bn_eval_fwd(hipStream_t st, int dtype, int M, int C, const void *x, const float *gamma,
                              const float *beta, const float *running_row, float *saved, void *out) {
  hipLaunchKernelGGL(k_bn_eval_prepare, dim3((C + kThreads - 1) / kThreads), dim3(kThreads), 0, st, C, running_row,
                     saved);
  dim3 agrid(blocks_for((long long)M * C, 4096), 1);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_bn_apply_relu<float>, agrid, dim3(kThreads), 0, st, M, C, (const float *)x, 0LL, gamma,
                                beta, 0LL, saved, (float *)out, 0LL),
             hipLaunchKernelGGL(k_bn_apply_relu<bf16_t>, agrid, dim3(kThreads), 0, st, M, C, (const bf16_t *)x, 0LL,
                                gamma, beta, 0LL, saved, (bf16_t *)out, 0LL));
  return hipGetLastError();
}

hipError_t launch_bn_bwd(hipStream_t st, int dtype, int n, int M, int C, const void *x, long long x_rs,
                         const void *dout, long long dout_rs, const float *gamma, const float *beta, long long p_rs,
                         const float *saved, double *partial, float *sums, float *dgamma, float *dbeta,
                         const void *add, long long add_rs, void *dx, long long dx_rs) {
  const int S = colreduce_splits(n, M), chunk = col_chunk(M, S), ct = channel_lanes(C);
  dim3 grid(S, n);
  DISPATCH_T(dtype,
             (run_colreduce<float, 2>(st, grid, M, C, chunk, ct, x, x_rs, dout, dout_rs, saved, gamma, beta, p_rs,
                                      partial)),
             (run_colreduce<bf16_t, 2>(st, grid, M, C, chunk, ct, x, x_rs, dout, dout_rs, saved, gamma, beta, p_rs,
                                       partial)));
  hipLaunchKernelGGL(k_bn_bwd_finalize, dim3(C, n), dim3(kFinThreads), 0, st, C, S, partial, sums, dgamma, dbeta, p_rs);
  const int vw = dtype ? 8 : 4;
  if (C % vw == 0 && x_rs % vw == 0 && dout_rs % vw == 0 && dx_rs % vw == 0 && add_rs % vw == 0 && aligned_to(x, 16) &&
      aligned_to(dout, 16) && aligned_to(dx, 16) && aligned_to(add, 16)) {
    dim3 vgrid(blocks_for((long long)M * (C / vw), 8192), n);
    DISPATCH_T(dtype,
               hipLaunchKernelGGL(k_bn_bwd_apply_vec<float>, vgrid, dim3(kThreads), 0, st, M, C, (const float *)x, x_rs,
                                  (const float *)dout, dout_rs, gamma, beta, p_rs, saved, sums, (const float *)add,
                                  add_rs, (float *)dx, dx_rs),
               hipLaunchKernelGGL(k_bn_bwd_apply_vec<bf16_t>, vgrid, dim3(kThreads), 0, st, M, C, (const bf16_t *)x, x_rs,
                                  (const bf16_t *)dout, dout_rs, gamma, beta, p_rs, saved, sums, (const bf16_t *)add,
                                  add_rs, (bf16_t *)dx, dx_rs));
    return hipGetLastError();
  }
  dim3 agrid(blocks_for((long long)M * C, 4096), n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_bn_bwd_apply<float>, agrid, dim3(kThreads), 0, st, M, C, (const float *)x, x_rs,
                                (const float *)dout, dout_rs, gamma, beta, p_rs, saved, sums, (const float *)add, add_rs,
                                (float *)dx, dx_rs),
             hipLaunchKernelGGL(k_bn_bwd_apply<bf16_t>, agrid, dim3(kThreads), 0, st, M, C, (const bf16_t *)x, x_rs,
                                (const bf16_t *)dout, dout_rs, gamma, beta, p_rs, saved, sums, (const bf16_t *)add,
                                add_rs, (bf16_t *)dx, dx_rs));
  return hipGetLastError();
}

hipError_t launch_weight_transpose(hipStream_t st, int dtype, int n, int Cout, int RS, int Cin, const void *w,
                                   long long w_rs, void *wt, long long wt_rs) {
  dim3 grid(blocks_for((long long)Cout * RS * Cin, 65535), n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_weight_transpose<float>, grid, dim3(kThreads), 0, st, Cout, RS, Cin, (const float *)w,
                                w_rs, (float *)wt, wt_rs),
             hipLaunchKernelGGL(k_weight_transpose<bf16_t>, grid, dim3(kThreads), 0, st, Cout, RS, Cin,
                                (const bf16_t *)w, w_rs, (bf16_t *)wt, wt_rs));
  return hipGetLastError();
}

bool transpose_vector_ok(int dtype, int cout, int cin, long long src_off) {
  const int vw = dtype ? 8 : 4;
  return cout % vw == 0 && cin % vw == 0 && src_off % vw == 0;
}

void transpose_table_finish(TransposeTable &tab) {
  tab.tile_begin[0] = 0;
  for (int i = 0; i < tab.count; ++i)
    tab.tile_begin[i + 1] = tab.tile_begin[i] + ((tab.cout[i] + 63) / 64) * ((tab.cin[i] + 63) / 64) * tab.rs[i];
}

hipError_t launch_weight_transpose_all(hipStream_t st, int dtype, int n, const TransposeTable &tab, const void *params,
                                       long long p_rs, void *dst_base) {
  if (tab.count < 1) return hipSuccess;
  if (tab.vec) {
    const int vw = dtype ? 8 : 4;
    if (p_rs % vw || !aligned_to(params, 16) || !aligned_to(dst_base, 16) || tab.tile_begin[tab.count] < 1)
      return hipErrorInvalidValue;
    dim3 vgrid(tab.tile_begin[tab.count], n);
    DISPATCH_T(dtype,
               hipLaunchKernelGGL(k_weight_transpose_vec<float>, vgrid, dim3(kThreads), 0, st, tab, (const float *)params,
                                  p_rs, (char *)dst_base),
               hipLaunchKernelGGL(k_weight_transpose_vec<bf16_t>, vgrid, dim3(kThreads), 0, st, tab,
                                  (const bf16_t *)params, p_rs, (char *)dst_base));
    return hipGetLastError();
  }
  dim3 grid(256, tab.count, n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_weight_transpose_all<float>, grid, dim3(kThreads), 0, st, tab, (const float *)params, p_rs,
                                (char *)dst_base),
             hipLaunchKernelGGL(k_weight_transpose_all<bf16_t>, grid, dim3(kThreads), 0, st, tab, (const bf16_t *)params,
                                p_rs, (char *)dst_base));
  return hipGetLastError();
}

hipError_t launch_dropout(hipStream_t st, int dtype, int n, long long count, const void *in, long long in_rs, void *out,
                          long long out_rs, const void *relu_src, long long relu_rs, unsigned seed,
                          const long long *step_dev, int site, unsigned thresh, float scale) {
  dim3 grid(blocks_for(count, 16384), n);
  DISPATCH_T(dtype,
             hipLaunchKernelGGL(k_dropout<float>, grid, dim3(kThreads), 0, st, count, (const float *)in, in_rs, (float *)out,
                                out_rs, (const float *)relu_src, relu_rs, seed, step_dev, (unsigned)site, thresh, scale),
             hipLaunchKernelGGL(k_dropout<bf16_t>, grid, dim3(kThreads), 0, st, count, (const bf16_t *)in, in_rs,
                                (bf16_t *)out, out_rs, (const bf16_t *)relu_src, relu_rs, seed, step_dev, (unsigned)site,
                                thresh, scale));
  return hipGetLastError();
}

hipError_t launch_convert(hipStream_t st, int dtype, const float *src, void *dst, long long count) {
  dim3 grid(blocks_for(count, 65535));
  DISPATCH_T(dtype, hipLaunchKernelGGL(k_convert<float>, grid, dim3(kThreads), 0, st, src, (float *)dst, count),
             hipLaunchKernelGGL(k_convert<bf16_t>, grid, dim3(kThreads), 0, st, src, (bf16_t *)dst, count));
  return hipGetLastError();
}

hipError_t launch_fill(hipStream_t st, float *dst, long long count, float value) {
  hipLaunchKernelGGL(k_fill, dim3(blocks_for(count, 65535)), dim3(kThreads), 0, st, dst, count, value);
  return hipGetLastError();
}

hipError_t launch_row_mean(hipStream_t st, int n, long long len, const float *in, long long rs, float *out) {
  hipLaunchKernelGGL(k_row_mean, dim3(blocks_for(len, 65535)), dim3(kThreads), 0, st, n, len, in, rs, out);
  return hipGetLastError();
}
