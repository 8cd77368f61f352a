// Layout kernels around the matrix-core passes: tiled transposes between the
// caller's NCHW / KCRS tensors and the batch-innermost work copies, plus the
// small set-up kernels (pixel ordering, fills, reductions).
#pragma once
#include "conv_common.h"
#include "pixel_order.h"

namespace cs {

// dst[b*dstBatch + l*dstPitch + n] = (n < rows && b < batchValid) ? src[b*srcBatch + n*srcPitch + l] : 0
// for 0 <= l < cols, 0 <= n < rowsPad, b = batch0 + blockIdx.z.  64x64 tiles through LDS,
// both sides coalesced.  grid = (ceil(cols/64), ceil(rowsPad/64), batches).  If zero_page is
// not null the first workgroup also clears its ZERO_PAGE_FLOATS floats (the page masked DMA
// lanes read).  Destination rows can be re-ordered: group > 0, interleave = 0 leaves one row
// free after every group rows (row l goes to l + l/group); group > 0, interleave > 0 reads l
// as (a, b) = (l / group, l % group) and writes row b*interleave + a.  Tin/Tout are float or
// uint16_t (bfloat16 bits).
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void transpose_in_kernel(
    const Tin* __restrict__ src, int64_t srcBatch, int64_t srcPitch, int rows, int cols,
    Tout* __restrict__ dst, int64_t dstBatch, int64_t dstPitch, int rowsPad, int batch0, int batchValid,
    float* __restrict__ zero_page, int group, int interleave) {
  __shared__ float tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int l0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
  if (zero_page && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
    for (int i = threadIdx.x; i < ZERO_PAGE_FLOATS; i += 256) zero_page[i] = 0.f;
  const int b = batch0 + blockIdx.z;
  const bool bok = b < batchValid;
  src += (int64_t)(bok ? b : 0) * srcBatch;
  dst += (int64_t)b * dstBatch;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int nn = ty + 4 * i;
    const int n = n0 + nn, l = l0 + tx;
    float v = 0.f;
    if (bok && n < rows && l < cols) v = load_as_f32<Tin>(src + (int64_t)n * srcPitch + l);
    tile[nn][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int ll = ty + 4 * i;
    const int l = l0 + ll, n = n0 + tx;
    const int lrow = group <= 0 ? l : interleave > 0 ? (l % group) * interleave + l / group : l + l / group;
    if (l < cols && n < rowsPad) store_from_f32<Tout>(dst + (int64_t)lrow * dstPitch + n, tile[tx][ll]);
  }
}

// The same when every address involved is a multiple of four elements (16 bytes for fp32, 8 for
// bfloat16) and cols, rowsPad and all pitches are multiples of four: four elements per global
// load and store, a quarter of the memory instructions.  Thread (tx, ty) = (t % 16, t / 16)
// loads columns 4*tx..+3 of rows ty, ty+16, .. and stores images 4*tx..+3 of destination rows
// ty, ty+16, ..
template <typename Tin, typename Tout>
__global__ __launch_bounds__(256) void transpose_in_v4_kernel(
    const Tin* __restrict__ src, int64_t srcBatch, int64_t srcPitch, int rows, int cols,
    Tout* __restrict__ dst, int64_t dstBatch, int64_t dstPitch, int rowsPad, int batch0, int batchValid,
    float* __restrict__ zero_page, int group, int interleave) {
  __shared__ float tile[64][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int l0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
  if (zero_page && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
    for (int i = threadIdx.x; i < ZERO_PAGE_FLOATS; i += 256) zero_page[i] = 0.f;
  const int b = batch0 + blockIdx.z;
  const bool bok = b < batchValid;
  src += (int64_t)(bok ? b : 0) * srcBatch;
  dst += (int64_t)b * dstBatch;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int nn = ty + 16 * i;
    const int n = n0 + nn, l = l0 + 4 * tx;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (bok && n < rows && l < cols) v = load4_as_f32<Tin>(src + (int64_t)n * srcPitch + l);
#pragma unroll
    for (int k = 0; k < 4; ++k) tile[nn][4 * tx + k] = v[k];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ll = ty + 16 * i;
    const int l = l0 + ll, n = n0 + 4 * tx;
    const int lrow = group <= 0 ? l : interleave > 0 ? (l % group) * interleave + l / group : l + l / group;
    if (l < cols && n < rowsPad) {
      f32x4 v;
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = tile[4 * tx + k][ll];
      store4_from_f32<Tout>(dst + (int64_t)lrow * dstPitch + n, v);
    }
  }
}

// dst[n*dstPitch + l] (+)= src[l*srcPitch + n] for 0 <= l < cols, 0 <= n < rows.
// grid = (ceil(cols/64), ceil(rows/64)).
template <typename Tout, bool ACC>
__global__ __launch_bounds__(256) void transpose_out_kernel(
    const float* __restrict__ src, int64_t srcPitch, int rows, int cols,
    Tout* __restrict__ dst, int64_t dstPitch) {
  __shared__ float tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int l0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int ll = ty + 4 * i;
    const int l = l0 + ll, n = n0 + tx;
    float v = 0.f;
    if (l < cols && n < rows) v = src[(int64_t)l * srcPitch + n];
    tile[ll][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int nn = ty + 4 * i;
    const int n = n0 + nn, l = l0 + tx;
    if (n < rows && l < cols) {
      Tout* p = dst + (int64_t)n * dstPitch + l;
      float v = tile[tx][nn];
      if (ACC) v += load_as_f32<Tout>(p);
      store_from_f32<Tout>(p, v);
    }
  }
}

// The same when every address is a multiple of four elements and cols and both pitches are
// multiples of four (rows may be ragged: the source rows are padded).
template <typename Tout, bool ACC>
__global__ __launch_bounds__(256) void transpose_out_v4_kernel(
    const float* __restrict__ src, int64_t srcPitch, int rows, int cols,
    Tout* __restrict__ dst, int64_t dstPitch) {
  __shared__ float tile[64][65];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int l0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ll = ty + 16 * i;
    const int l = l0 + ll, n = n0 + 4 * tx;   // srcPitch covers the padded batch: a whole vector is readable
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (l < cols && n < srcPitch) v = *(const f32x4*)(src + (int64_t)l * srcPitch + n);
#pragma unroll
    for (int k = 0; k < 4; ++k) tile[ll][4 * tx + k] = v[k];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int nn = ty + 16 * i;
    const int n = n0 + nn, l = l0 + 4 * tx;
    if (n < rows && l < cols) {
      Tout* p = dst + (int64_t)n * dstPitch + l;
      f32x4 v;
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = tile[4 * tx + k][nn];
      if (ACC) {
        const f32x4 o = load4_as_f32<Tout>(p);
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] += o[k];
      }
      store4_from_f32<Tout>(p, v);
    }
  }
}

// Input gradient of layers with few input channels, second step.  The matrix-core step
// leaves T[(c,r,s)][p][q][n] = sum_k w[k,c,r,s] * dy[n,k,p,q]; every input pixel (h,v)
// collects the (r,s,p,q) combinations whose window position lands on it:
//   dx[n][c][h][v] (+)= sum_{r,s : p*sh-ph+r = h, q*sw-pw+s = v} T[(c,r,s)][p][q][n]
// in increasing (r,s) order.  A workgroup owns 16 consecutive (c,h,v) positions and 64 images:
// a wavefront reads T rows along n (coalesced), the tile is turned in LDS and written out along
// (c,h,v).  The tap loops are branch free (a miss reads a clamped element and adds a selected
// zero), so that the loads of several taps are in flight together.
// grid = (ceil(C*H*W/16), ceil(N/64)).
constexpr int COL2IM_ROWS = 16;
template <typename Tout, bool ACC>
__global__ __launch_bounds__(256) void col2im_out_kernel(Geo g, const float* __restrict__ T,
                                                         Tout* __restrict__ dx) {
  __shared__ float tile[COL2IM_ROWS][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int l0 = blockIdx.x * COL2IM_ROWS, n0 = blockIdx.y * 64;
  const int CHW = g.C * g.HW;
#pragma unroll 1
  for (int i = 0; i < COL2IM_ROWS / 4; ++i) {
    const int ll = ty + 4 * i;
    const int l = l0 + ll, n = n0 + tx;
    float acc = 0.f;
    if (l < CHW && n < g.Np) {
      const int c = l / g.HW, hw = l - c * g.HW;
      const int h = hw / g.W, v = hw - h * g.W;
      const float* Tc = T + (int64_t)c * g.RS * g.PQ * g.Np + n;
      // only taps r = (h+ph) mod sh, +sh, ... can have h+ph-r divisible by the stride (same for s)
      for (int r = (h + g.ph) % g.sh; r < g.R; r += g.sh) {
        const int hr = h + g.ph - r;
        const int p = hr / g.sh;
        const bool rok = hr >= 0 && p < g.P;
        const int pc = rok ? p : 0;
#pragma unroll 5
        for (int s = (v + g.pw) % g.sw; s < g.S; s += g.sw) {
          const int vs = v + g.pw - s;
          const int q = vs / g.sw;
          const bool ok = rok && vs >= 0 && q < g.Q;
          const float t = Tc[((int64_t)(r * g.S + s) * g.PQ + pc * g.Q + (ok ? q : 0)) * g.Np];
          acc += ok ? t : 0.f;
        }
      }
    }
    tile[ll][tx] = acc;
  }
  __syncthreads();
  const int wl = threadIdx.x & (COL2IM_ROWS - 1), wn = threadIdx.x / COL2IM_ROWS;
#pragma unroll
  for (int i = 0; i < 64 / (256 / COL2IM_ROWS); ++i) {
    const int nn = wn + (256 / COL2IM_ROWS) * i;
    const int n = n0 + nn, l = l0 + wl;
    if (n < g.N && l < CHW) {
      Tout* p = dx + (int64_t)n * CHW + l;
      float v = tile[wl][nn];
      if (ACC) v += load_as_f32<Tout>(p);
      store_from_f32<Tout>(p, v);
    }
  }
}

// dst[r*dstPitch + c] = c < cols ? src[r*srcPitch + c] : 0 for c < dstPitch: rows of
// the filter matrix converted to fp32 and re-pitched to a multiple of 4.
template <typename Tin>
__global__ __launch_bounds__(256) void repitch_rows_kernel(
    const Tin* __restrict__ src, int64_t srcPitch, int rows, int cols,
    float* __restrict__ dst, int dstPitch) {
  const int64_t total = (int64_t)rows * dstPitch;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int r = (int)(i / dstPitch), c = (int)(i - (int64_t)r * dstPitch);
    dst[i] = c < cols ? load_as_f32<Tin>(src + (int64_t)r * srcPitch + c) : 0.f;
  }
}

// bf16 filters w[k][c][rs] -> w_krsc[k][rs][Cp] (channels innermost, zero for C <= c < Cp).
// A workgroup takes 64 channels of one kernel: their 64*RS elements are contiguous in w, and
// each tap's 64 channels are contiguous in the result.  grid = (ceil(Cp/64), Ks); taps in
// rounds of 64 so that the LDS tile stays at 16 KB.
__global__ __launch_bounds__(256) void filters_to_krsc_kernel(const uint16_t* __restrict__ w, int C, int RS, int Cp,
                                                              uint16_t* __restrict__ out) {
  __shared__ uint16_t tile[64 * 65];   // [channel][tap of the round], pitch 65
  const int c0 = blockIdx.x * 64, k = blockIdx.y;
  const uint16_t* wk = w + (int64_t)k * C * RS;
  uint16_t* ok = out + (int64_t)k * RS * Cp;
  for (int t0 = 0; t0 < RS; t0 += 64) {
    const int nt = min(64, RS - t0);
    // read: thread -> (channel, tap) with taps fastest, as they lie in memory
    for (int e = threadIdx.x; e < 64 * nt; e += 256) {
      const int c = e / nt, t = e - c * nt;
      tile[c * 65 + t] = c0 + c < C ? wk[(int64_t)(c0 + c) * RS + t0 + t] : (uint16_t)0;
    }
    __syncthreads();
    // write: thread -> (tap, channel) with channels fastest
    for (int e = threadIdx.x; e < 64 * nt; e += 256) {
      const int t = e >> 6, c = e & 63;
      if (c0 + c < Cp) ok[(int64_t)(t0 + t) * Cp + c0 + c] = tile[c * 65 + t];
    }
    __syncthreads();
  }
}

// Forward pass: for reduction index kk = (c,r,s), tab[kk] = byte offset of that tap inside
// x_t relative to a pixel's window origin, counted from the zero page in front of x_t, and
// tab[entries + kk] = (r<<16)|s.  Entries past C*R*S repeat entry 0: the filter operand is
// zero there, so any finite input value will do.
__global__ void fwd_tap_table_kernel(Geo g, int entries, int* __restrict__ tab) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= entries) return;
  const int kk = i < g.CRS ? i : 0;
  const int c = kk / g.RS, rs = kk - c * g.RS;
  const int r = rs / g.S, s = rs - r * g.S;
  tab[i] = (int)(((unsigned)((c * g.HW + r * g.W + s) * g.Np) + (unsigned)ZERO_PAGE_FLOATS) * 4u);
  tab[entries + i] = (r << 16) | s;
}

// One workgroup runs the phases of pixel_order.h: perm[position] = pixel, pixels by decreasing
// tap count, and (with `pre`) the line of the CT column tiles of bpt blocks each.  scratch holds
// po::axes_ints(H, W) ints, used when the per-axis tables do not fit in LDS.  Launch with
// po::THREADS threads.
__global__ __launch_bounds__(po::THREADS) void bwd_data_pixel_order_kernel(Geo g, int* __restrict__ perm,
                                                                           int* __restrict__ scratch, int CT, int nkc,
                                                                           int bpt, int* __restrict__ pre) {
  __shared__ int bins[po::BINS], rowCnt[po::AXIS_CNT], colCnt[po::AXIS_CNT], part[po::THREADS];
  __shared__ int s_axes[po::AXES_LDS];
  po::Tables<int*> t;
  t.bins = bins; t.rowCnt = rowCnt; t.colCnt = colCnt; t.part = part;
  t.axes = po::axes_ints(g.H, g.W) <= po::AXES_LDS ? s_axes : scratch;
  t.perm = perm; t.pre = pre;
  const int tid = threadIdx.x, T = po::THREADS;
  po::phase_axes(g, t, tid, T);
  __threadfence_block();
  __syncthreads();
  po::phase_ranks(g, t, tid, T);
  __threadfence_block();
  __syncthreads();
  po::phase_bins(g, t, tid, T);
  __syncthreads();
  po::phase_scan_bins(g, t, tid, T);
  __syncthreads();
  po::phase_place(g, t, tid, T);
  if (pre == nullptr) return;
  __threadfence_block();
  __syncthreads();
  po::phase_lengths(g, t, CT, nkc, bpt, tid, T);
  __syncthreads();
  for (int d = 1; d < T; d <<= 1) {   // part[] becomes its inclusive running sum
    const int v = tid >= d ? part[tid - d] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  po::phase_prefix(t, CT, tid, T);
}

template <typename T>
__global__ __launch_bounds__(256) void fill_zero_kernel(T* __restrict__ p, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
       i += (int64_t)gridDim.x * blockDim.x)
    p[i] = (T)0;
}

// Clears `rows` runs of `len` floats that start `stride` floats apart.
__global__ __launch_bounds__(256) void fill_zero_rows_kernel(float* __restrict__ p, int64_t stride, int rows, int len) {
  const int64_t total = (int64_t)rows * len;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int r = (int)(i / len);
    p[(int64_t)r * stride + (i - (int64_t)r * len)] = 0.f;
  }
}

// dw[i] = sum_z part[z*stride + i], summed in increasing z (bit-stable).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(
    const float* __restrict__ part, int64_t stride, int splits, float* __restrict__ dw, int64_t count) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
       i += (int64_t)gridDim.x * blockDim.x) {
    float acc = part[i];
#pragma unroll 8
    for (int z = 1; z < splits; ++z) acc += part[(int64_t)z * stride + i];
    dw[i] = acc;
  }
}

}  // namespace cs
