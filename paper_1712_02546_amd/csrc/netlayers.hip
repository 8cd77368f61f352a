// netlayers.hip -- the network's layers other than the convolutions (Section 4.1): channel
// normalisation, max pooling, fully connected layer, softmax loss, gradient step.  All of them
// are bound by memory traffic; the kernels are plain, coalesced along the innermost index,
// free of atomics (fixed summation orders) and launched over the whole tensor.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "../../include/convnet.h"

namespace {

constexpr int kThreads = 256;
constexpr int64_t kMaxCount = ((int64_t)1 << 31) - 1;

inline int blocks_for(int64_t count) { return (int)std::min<int64_t>((count + kThreads - 1) / kThreads, 65536); }
inline int launch_status() { return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ERR_LAUNCH; }

// ---- normalisation ---------------------------------------------------------------------
// s^p for s > 0 through the hardware's base-2 logarithm and exponential (relative error about
// 1e-6 for the exponents and scales that occur here, far inside the layer's tolerance).
__device__ __forceinline__ float pow_pos(float s, float p) { return __builtin_amdgcn_exp2f(p * __builtin_amdgcn_logf(s)); }

// grid = (ceil(C*HW/kThreads), N): one 32-bit division per thread.
__global__ __launch_bounds__(kThreads) void norm_fwd_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                            float* __restrict__ scale, int C, int HW, int half,
                                                            float kappa, float alpha, float beta) {
  const unsigned ci = blockIdx.x * kThreads + threadIdx.x;
  if (ci >= (unsigned)(C * HW)) return;
  const int c = (int)(ci / (unsigned)HW), i = (int)(ci - (unsigned)c * (unsigned)HW);
  const float* xn = x + (int64_t)blockIdx.y * C * HW + i;
  const int lo = max(0, c - half), hi = min(C, c + half + 1);
  float ss = 0.f;
  for (int cc = lo; cc < hi; ++cc) {
    const float v = xn[(int64_t)cc * HW];
    ss += v * v;
  }
  const float s = kappa + alpha * ss;
  const int64_t e = (int64_t)blockIdx.y * C * HW + ci;
  scale[e] = s;
  y[e] = x[e] * pow_pos(s, -beta);
}

// Four neighbouring pixels per thread (HW a multiple of four, 16-byte aligned tensors): 16-byte loads and stores.
typedef float f32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(kThreads) void norm_fwd_v4_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                               float* __restrict__ scale, int C, int HW, int half,
                                                               float kappa, float alpha, float beta) {
  const unsigned ci = (blockIdx.x * kThreads + threadIdx.x) * 4u;
  if (ci >= (unsigned)(C * HW)) return;
  const int c = (int)(ci / (unsigned)HW), i = (int)(ci - (unsigned)c * (unsigned)HW);
  const float* xn = x + (int64_t)blockIdx.y * C * HW + i;
  const int lo = max(0, c - half), hi = min(C, c + half + 1);
  f32x4 ss = {0.f, 0.f, 0.f, 0.f};
  for (int cc = lo; cc < hi; ++cc) {
    const f32x4 v = *(const f32x4*)(xn + (int64_t)cc * HW);
    ss += v * v;
  }
  const int64_t e = (int64_t)blockIdx.y * C * HW + ci;
  const f32x4 xe = *(const f32x4*)(x + e);
  f32x4 s, o;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    s[k] = kappa + alpha * ss[k];
    o[k] = xe[k] * pow_pos(s[k], -beta);
  }
  *(f32x4*)(scale + e) = s;
  *(f32x4*)(y + e) = o;
}

__global__ __launch_bounds__(kThreads) void norm_bwd_v4_kernel(const float* __restrict__ x, const float* __restrict__ y,
                                                               const float* __restrict__ scale,
                                                               const float* __restrict__ dy, float* __restrict__ dx, int C,
                                                               int HW, int half, float alpha, float beta) {
  const unsigned ci = (blockIdx.x * kThreads + threadIdx.x) * 4u;
  if (ci >= (unsigned)(C * HW)) return;
  const int c = (int)(ci / (unsigned)HW), i = (int)(ci - (unsigned)c * (unsigned)HW);
  const int64_t base = (int64_t)blockIdx.y * C * HW + i;
  const int lo = max(0, c - half), hi = min(C, c + half + 1);
  f32x4 t = {0.f, 0.f, 0.f, 0.f};
  for (int cc = lo; cc < hi; ++cc) {
    const int64_t j = base + (int64_t)cc * HW;
    const f32x4 a = *(const f32x4*)(dy + j), b = *(const f32x4*)(y + j), d = *(const f32x4*)(scale + j);
#pragma unroll
    for (int k = 0; k < 4; ++k) t[k] += a[k] * b[k] / d[k];
  }
  const int64_t e = base + (int64_t)c * HW;
  const f32x4 de = *(const f32x4*)(dy + e), se = *(const f32x4*)(scale + e), xe = *(const f32x4*)(x + e);
  f32x4 o;
#pragma unroll
  for (int k = 0; k < 4; ++k) o[k] = de[k] * pow_pos(se[k], -beta) - 2.f * alpha * beta * xe[k] * t[k];
  *(f32x4*)(dx + e) = o;
}

// dy[c']*x[c']*scale[c']^(-beta-1) = dy[c']*y[c']/scale[c'], so the window sum needs no power function.
__global__ __launch_bounds__(kThreads) void norm_bwd_kernel(const float* __restrict__ x, const float* __restrict__ y,
                                                            const float* __restrict__ scale, const float* __restrict__ dy,
                                                            float* __restrict__ dx, int C, int HW, int half, float alpha,
                                                            float beta) {
  const unsigned ci = blockIdx.x * kThreads + threadIdx.x;
  if (ci >= (unsigned)(C * HW)) return;
  const int c = (int)(ci / (unsigned)HW), i = (int)(ci - (unsigned)c * (unsigned)HW);
  const int64_t base = (int64_t)blockIdx.y * C * HW + i;
  const int lo = max(0, c - half), hi = min(C, c + half + 1);
  float t = 0.f;
  for (int cc = lo; cc < hi; ++cc) {
    const int64_t j = base + (int64_t)cc * HW;
    t += dy[j] * y[j] / scale[j];
  }
  const int64_t e = base + (int64_t)c * HW;
  dx[e] = dy[e] * pow_pos(scale[e], -beta) - 2.f * alpha * beta * x[e] * t;
}

// ---- max pooling -----------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void pool_fwd_kernel(const float* __restrict__ x, float* __restrict__ y, int H,
                                                            int W, int P, int Q, int win, int stride, int64_t count) {
  // counts are below 2^31: unsigned 32-bit divisions
  for (int64_t e64 = (int64_t)blockIdx.x * kThreads + threadIdx.x; e64 < count; e64 += (int64_t)gridDim.x * kThreads) {
    const unsigned e = (unsigned)e64;
    const unsigned m = e / (unsigned)(P * Q), pq = e - m * (unsigned)(P * Q);
    const int p = (int)(pq / (unsigned)Q), q = (int)(pq - (unsigned)p * (unsigned)Q);
    const float* xm = x + (int64_t)m * H * W + (int64_t)(p * stride) * W + q * stride;
    float best = xm[0];
    for (int i = 0; i < win; ++i)
      for (int j = 0; j < win; ++j) best = fmaxf(best, xm[i * W + j]);
    y[e64] = best;
  }
}

// Gather form: every input element looks at the windows that contain it and takes dy from those
// whose first maximum it is.
__global__ __launch_bounds__(kThreads) void pool_bwd_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                            float* __restrict__ dx, int H, int W, int P, int Q, int win,
                                                            int stride, int64_t count) {
  for (int64_t e64 = (int64_t)blockIdx.x * kThreads + threadIdx.x; e64 < count; e64 += (int64_t)gridDim.x * kThreads) {
    const unsigned e = (unsigned)e64;
    const unsigned mm = e / (unsigned)(H * W), hw = e - mm * (unsigned)(H * W);
    const int h = (int)(hw / (unsigned)W), w = (int)(hw - (unsigned)h * (unsigned)W);
    const int64_t m = mm;
    const float* xm = x + m * H * W;
    const float mine = xm[h * W + w];
    // windows p with p*stride <= h < p*stride + win
    const int p0 = max(0, (h - win + stride) / stride), p1 = min(P - 1, h / stride);
    const int q0 = max(0, (w - win + stride) / stride), q1 = min(Q - 1, w / stride);
    float acc = 0.f;
    for (int p = p0; p <= p1; ++p)
      for (int q = q0; q <= q1; ++q) {
        // is (h,w) the first maximum of window (p,q)?
        bool first = true;
        for (int i = 0; i < win && first; ++i)
          for (int j = 0; j < win; ++j) {
            const int hh = p * stride + i, ww = q * stride + j;
            const float v = xm[hh * W + ww];
            const bool before = hh < h || (hh == h && ww < w);
            if (v > mine || (before && v == mine)) {
              first = false;
              break;
            }
          }
        if (first) acc += dy[m * P * Q + (int64_t)p * Q + q];
      }
    dx[e64] = acc;
  }
}

// Windows that tile the image exactly (win = stride = 2, H = 2P, W = 2Q): a thread owns one window, finds its first
// maximum and writes the window's four gradients.
__global__ __launch_bounds__(kThreads) void pool_bwd_2x2_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                                float* __restrict__ dx, int W, int P, int Q, int64_t count) {
  for (int64_t e64 = (int64_t)blockIdx.x * kThreads + threadIdx.x; e64 < count; e64 += (int64_t)gridDim.x * kThreads) {
    const unsigned e = (unsigned)e64;
    const unsigned m = e / (unsigned)(P * Q), pq = e - m * (unsigned)(P * Q);
    const int p = (int)(pq / (unsigned)Q), q = (int)(pq - (unsigned)p * (unsigned)Q);
    const int64_t o = (int64_t)m * (4 * P * Q) + (int64_t)(2 * p) * W + 2 * q;
    const float2 top = *(const float2*)(x + o), bot = *(const float2*)(x + o + W);
    int arg = 0;
    float best = top.x;
    if (top.y > best) { best = top.y; arg = 1; }
    if (bot.x > best) { best = bot.x; arg = 2; }
    if (bot.y > best) { best = bot.y; arg = 3; }
    const float g = dy[e64];
    *(float2*)(dx + o) = make_float2(arg == 0 ? g : 0.f, arg == 1 ? g : 0.f);
    *(float2*)(dx + o + W) = make_float2(arg == 2 ? g : 0.f, arg == 3 ? g : 0.f);
  }
}

// ---- fully connected -------------------------------------------------------------------
constexpr int kOB = 8;   // outputs per workgroup / thread block of outputs

// grid (N, ceil(O/kOB)): a workgroup forms kOB dot products of length I for one image.
constexpr int kFcThreads = 1024;   // many loads in flight per compute unit: the dot products are latency bound
__global__ __launch_bounds__(kFcThreads) void fc_fwd_kernel(const float* __restrict__ x, const float* __restrict__ W,
                                                            const float* __restrict__ b, float* __restrict__ y, int I,
                                                            int O) {
  __shared__ float red[kOB][kFcThreads];
  const int n = blockIdx.x, o0 = blockIdx.y * kOB;
  const float* xn = x + (int64_t)n * I;
  float acc[kOB];
#pragma unroll
  for (int k = 0; k < kOB; ++k) acc[k] = 0.f;
#pragma unroll 2
  for (int i = threadIdx.x; i < I; i += kFcThreads) {
    const float v = xn[i];
#pragma unroll
    for (int k = 0; k < kOB; ++k)
      if (o0 + k < O) acc[k] += v * W[(int64_t)(o0 + k) * I + i];
  }
#pragma unroll
  for (int k = 0; k < kOB; ++k) red[k][threadIdx.x] = acc[k];
  __syncthreads();
  for (int s = kFcThreads / 2; s > 0; s >>= 1) {   // fixed tree: the same order on every run
    if (threadIdx.x < s)
#pragma unroll
      for (int k = 0; k < kOB; ++k) red[k][threadIdx.x] += red[k][threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x < kOB && o0 + threadIdx.x < O)
    y[(int64_t)n * O + o0 + threadIdx.x] = red[threadIdx.x][0] + (b ? b[o0 + threadIdx.x] : 0.f);
}

__global__ __launch_bounds__(kThreads) void fc_bwd_data_kernel(const float* __restrict__ W, const float* __restrict__ dy,
                                                               float* __restrict__ dx, int I, int O, int64_t count) {
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < count; e += (int64_t)gridDim.x * kThreads) {
    const int i = (int)(e % I);
    const int64_t n = e / I;
    float acc = 0.f;
    for (int o = 0; o < O; ++o) acc += dy[n * O + o] * W[(int64_t)o * I + i];
    dx[e] = acc;
  }
}

// grid (ceil(I/kFcWThreads), ceil(O/kOB)): a thread owns input i and kOB outputs, sums over the batch in order.
// Small workgroups so that a few thousand inputs already fill the chip; the batch loop is unrolled to keep
// several loads in flight per thread.
constexpr int kFcWThreads = 64;
__global__ __launch_bounds__(kFcWThreads) void fc_bwd_weight_kernel(const float* __restrict__ x, const float* __restrict__ dy,
                                                                    float* __restrict__ dW, int N, int I, int O) {
  const int i = blockIdx.x * kFcWThreads + threadIdx.x, o0 = blockIdx.y * kOB;
  if (i >= I) return;
  float acc[kOB];
#pragma unroll
  for (int k = 0; k < kOB; ++k) acc[k] = 0.f;
#pragma unroll 8
  for (int n = 0; n < N; ++n) {
    const float v = x[(int64_t)n * I + i];
#pragma unroll
    for (int k = 0; k < kOB; ++k)
      if (o0 + k < O) acc[k] += dy[(int64_t)n * O + o0 + k] * v;
  }
#pragma unroll
  for (int k = 0; k < kOB; ++k)
    if (o0 + k < O) dW[(int64_t)(o0 + k) * I + i] = acc[k];
}

__global__ __launch_bounds__(kThreads) void fc_bwd_bias_kernel(const float* __restrict__ dy, float* __restrict__ db, int N,
                                                               int O) {
  const int o = blockIdx.x * kThreads + threadIdx.x;
  if (o >= O) return;
  float acc = 0.f;
  for (int n = 0; n < N; ++n) acc += dy[(int64_t)n * O + o];
  db[o] = acc;
}

// ---- softmax loss ----------------------------------------------------------------------
__device__ __forceinline__ void row_max_and_sum(const float* zr, int O, float& mx, float& sum) {
  mx = zr[0];
  for (int o = 1; o < O; ++o) mx = fmaxf(mx, zr[o]);
  sum = 0.f;
  for (int o = 0; o < O; ++o) sum += expf(zr[o] - mx);
}

// One workgroup: per-image losses by its threads, then a fixed tree over the threads' partial sums.
__global__ __launch_bounds__(kThreads) void softmax_loss_fwd_kernel(const float* __restrict__ z,
                                                                    const int32_t* __restrict__ labels,
                                                                    float* __restrict__ loss, int N, int O) {
  __shared__ float red[kThreads];
  float acc = 0.f;
  for (int n = threadIdx.x; n < N; n += kThreads) {
    const float* zr = z + (int64_t)n * O;
    float mx, sum;
    row_max_and_sum(zr, O, mx, sum);
    acc += logf(sum) + mx - zr[labels[n]];
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = kThreads / 2; s > 0; s >>= 1) {
    if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = red[0] / (float)N;
}

__global__ __launch_bounds__(kThreads) void softmax_loss_bwd_kernel(const float* __restrict__ z,
                                                                    const int32_t* __restrict__ labels,
                                                                    float* __restrict__ dz, int N, int O) {
  const int n = blockIdx.x * kThreads + threadIdx.x;
  if (n >= N) return;
  const float* zr = z + (int64_t)n * O;
  float mx, sum;
  row_max_and_sum(zr, O, mx, sum);
  const float inv = 1.f / (float)N;
  const int lab = labels[n];
  // softmax - 1 at the label is minus the other classes' share; formed from their sum, it keeps
  // its relative accuracy when the label's probability is close to one
  float others = 0.f;
  for (int o = 0; o < O; ++o)
    if (o != lab) others += expf(zr[o] - mx);
  for (int o = 0; o < O; ++o)
    dz[(int64_t)n * O + o] = (o == lab ? -others / sum : expf(zr[o] - mx) / sum) * inv;
}

__global__ __launch_bounds__(kThreads) void sgd_kernel(float* __restrict__ w, const float* __restrict__ dw, float lr,
                                                       int64_t count) {
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < count; e += (int64_t)gridDim.x * kThreads)
    w[e] -= lr * dw[e];
}

}  // namespace

extern "C" {

int net_norm_fwd(const float* x, float* y, float* scale, int32_t N, int32_t C, int32_t HW, int32_t size, float kappa,
                 float alpha, float beta, void* hip_stream) {
  if (!x || !y || !scale) return CONV_ERR_NULL;
  if (N < 1 || C < 1 || HW < 1 || size < 1 || size % 2 == 0 || N > 65535) return CONV_ERR_SHAPE;
  const int64_t count = (int64_t)N * C * HW;
  if (count > kMaxCount) return CONV_ERR_SHAPE;
  if (HW % 4 == 0 && ((uintptr_t)x | (uintptr_t)y | (uintptr_t)scale) % 16 == 0)
    hipLaunchKernelGGL(norm_fwd_v4_kernel, dim3((unsigned)(((int64_t)C * HW / 4 + kThreads - 1) / kThreads), N),
                       dim3(kThreads), 0, (hipStream_t)hip_stream, x, y, scale, C, HW, size / 2, kappa, alpha, beta);
  else
    hipLaunchKernelGGL(norm_fwd_kernel, dim3((unsigned)(((int64_t)C * HW + kThreads - 1) / kThreads), N), dim3(kThreads),
                       0, (hipStream_t)hip_stream, x, y, scale, C, HW, size / 2, kappa, alpha, beta);
  return launch_status();
}

int net_norm_bwd(const float* x, const float* y, const float* scale, const float* dy, float* dx, int32_t N, int32_t C,
                 int32_t HW, int32_t size, float kappa, float alpha, float beta, void* hip_stream) {
  (void)kappa;   // already inside scale
  if (!x || !y || !scale || !dy || !dx) return CONV_ERR_NULL;
  if (N < 1 || C < 1 || HW < 1 || size < 1 || size % 2 == 0 || N > 65535) return CONV_ERR_SHAPE;
  const int64_t count = (int64_t)N * C * HW;
  if (count > kMaxCount) return CONV_ERR_SHAPE;
  if (HW % 4 == 0 && ((uintptr_t)x | (uintptr_t)y | (uintptr_t)scale | (uintptr_t)dy | (uintptr_t)dx) % 16 == 0)
    hipLaunchKernelGGL(norm_bwd_v4_kernel, dim3((unsigned)(((int64_t)C * HW / 4 + kThreads - 1) / kThreads), N),
                       dim3(kThreads), 0, (hipStream_t)hip_stream, x, y, scale, dy, dx, C, HW, size / 2, alpha, beta);
  else
    hipLaunchKernelGGL(norm_bwd_kernel, dim3((unsigned)(((int64_t)C * HW + kThreads - 1) / kThreads), N), dim3(kThreads),
                       0, (hipStream_t)hip_stream, x, y, scale, dy, dx, C, HW, size / 2, alpha, beta);
  return launch_status();
}

static int pool_dims(int32_t NC, int32_t H, int32_t W, int32_t win, int32_t stride, int& P, int& Q) {
  if (NC < 1 || H < 1 || W < 1 || win < 1 || stride < 1 || win > H || win > W) return CONV_ERR_SHAPE;
  P = (H - win) / stride + 1;
  Q = (W - win) / stride + 1;
  if ((int64_t)NC * H * W > kMaxCount) return CONV_ERR_SHAPE;
  return CONV_OK;
}

int net_pool_fwd(const float* x, float* y, int32_t NC, int32_t H, int32_t W, int32_t win, int32_t stride,
                 void* hip_stream) {
  if (!x || !y) return CONV_ERR_NULL;
  int P, Q;
  const int rc = pool_dims(NC, H, W, win, stride, P, Q);
  if (rc != CONV_OK) return rc;
  const int64_t count = (int64_t)NC * P * Q;
  hipLaunchKernelGGL(pool_fwd_kernel, dim3(blocks_for(count)), dim3(kThreads), 0, (hipStream_t)hip_stream, x, y, H, W,
                     P, Q, win, stride, count);
  return launch_status();
}

int net_pool_bwd(const float* x, const float* dy, float* dx, int32_t NC, int32_t H, int32_t W, int32_t win,
                 int32_t stride, void* hip_stream) {
  if (!x || !dy || !dx) return CONV_ERR_NULL;
  int P, Q;
  const int rc = pool_dims(NC, H, W, win, stride, P, Q);
  if (rc != CONV_OK) return rc;
  if (win == 2 && stride == 2 && H == 2 * P && W == 2 * Q && ((uintptr_t)x | (uintptr_t)dx) % 8 == 0) {
    const int64_t windows = (int64_t)NC * P * Q;
    hipLaunchKernelGGL(pool_bwd_2x2_kernel, dim3(blocks_for(windows)), dim3(kThreads), 0, (hipStream_t)hip_stream, x, dy,
                       dx, W, P, Q, windows);
    return launch_status();
  }
  const int64_t count = (int64_t)NC * H * W;
  hipLaunchKernelGGL(pool_bwd_kernel, dim3(blocks_for(count)), dim3(kThreads), 0, (hipStream_t)hip_stream, x, dy, dx, H,
                     W, P, Q, win, stride, count);
  return launch_status();
}

int net_fc_fwd(const float* x, const float* W, const float* b, float* y, int32_t N, int32_t I, int32_t O,
               void* hip_stream) {
  if (!x || !W || !y) return CONV_ERR_NULL;
  if (N < 1 || I < 1 || O < 1 || N > 65535 || (int64_t)N * I > kMaxCount || (int64_t)O * I > kMaxCount)
    return CONV_ERR_SHAPE;
  hipLaunchKernelGGL(fc_fwd_kernel, dim3(N, (O + kOB - 1) / kOB), dim3(kFcThreads), 0, (hipStream_t)hip_stream, x, W, b, y,
                     I, O);
  return launch_status();
}

int net_fc_bwd(const float* x, const float* W, const float* dy, float* dx, float* dW, float* db, int32_t N, int32_t I,
               int32_t O, void* hip_stream) {
  if (!dy || (dx && !W) || (dW && !x)) return CONV_ERR_NULL;
  if (N < 1 || I < 1 || O < 1 || (int64_t)N * I > kMaxCount || (int64_t)O * I > kMaxCount) return CONV_ERR_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (dx) {
    const int64_t count = (int64_t)N * I;
    hipLaunchKernelGGL(fc_bwd_data_kernel, dim3(blocks_for(count)), dim3(kThreads), 0, st, W, dy, dx, I, O, count);
  }
  if (dW)
    hipLaunchKernelGGL(fc_bwd_weight_kernel, dim3((I + kFcWThreads - 1) / kFcWThreads, (O + kOB - 1) / kOB), dim3(kFcWThreads), 0,
                       st, x, dy, dW, N, I, O);
  if (db) hipLaunchKernelGGL(fc_bwd_bias_kernel, dim3((O + kThreads - 1) / kThreads), dim3(kThreads), 0, st, dy, db, N, O);
  return launch_status();
}

int net_softmax_loss_fwd(const float* z, const int32_t* labels, float* loss, int32_t N, int32_t O, void* hip_stream) {
  if (!z || !labels || !loss) return CONV_ERR_NULL;
  if (N < 1 || O < 1 || (int64_t)N * O > kMaxCount) return CONV_ERR_SHAPE;
  hipLaunchKernelGGL(softmax_loss_fwd_kernel, dim3(1), dim3(kThreads), 0, (hipStream_t)hip_stream, z, labels, loss, N, O);
  return launch_status();
}

int net_softmax_loss_bwd(const float* z, const int32_t* labels, float* dz, int32_t N, int32_t O, void* hip_stream) {
  if (!z || !labels || !dz) return CONV_ERR_NULL;
  if (N < 1 || O < 1 || (int64_t)N * O > kMaxCount) return CONV_ERR_SHAPE;
  hipLaunchKernelGGL(softmax_loss_bwd_kernel, dim3((N + kThreads - 1) / kThreads), dim3(kThreads), 0,
                     (hipStream_t)hip_stream, z, labels, dz, N, O);
  return launch_status();
}

int net_sgd_update(float* w, const float* dw, float lr, int64_t count, void* hip_stream) {
  if (!w || !dw) return CONV_ERR_NULL;
  if (count < 0) return CONV_ERR_SHAPE;
  if (count == 0) return CONV_OK;
  hipLaunchKernelGGL(sgd_kernel, dim3(blocks_for(count)), dim3(kThreads), 0, (hipStream_t)hip_stream, w, dw, lr, count);
  return launch_status();
}

}  // extern "C"
