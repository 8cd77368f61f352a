// Pixel-major passes for layers with few input channels (first layers: C = 3).
//
// There the input x is tiny next to y / dy (cfg2: 1.6 MB against 200 MB), so the layout of
// the GEMM is chosen for y and dy: a 32-lane column block is 32 consecutive output pixels of
// one image, i.e. 128 contiguous bytes of the caller's NCHW tensor.  y is written and dy is
// read in place -- no batch-innermost work copy of either -- and the im2col side, which is
// a gather in this mapping, is staged with 4-byte LDS-DMA loads whose lane offsets are
// constants (a lane is one pixel, or one filter tap) while the tap (or pixel) moves in a
// scalar base register.  Out-of-image taps never need a test: when the layer has padding,
// x is first copied once into a zero-bordered fp32 image xb[N][C][Hp][Wp] (a few MB).
//
//   fwd         y_n[k][pix]   = sum_j  w[k][j]      * x_n[tap j at pix]      M = Ks, red = C*R*S
//   bwd_data    T_n[j][pix]   = sum_k  w[k][j]      * dy_n[k][pix]           M = C*R*S, red = Ks
//               dx_n[c][h][v] = sum of the T_n[(c,r,s)][pix] whose window tap lands on (h,v)
//   bwd_weight  dw[k][j]      = sum_(n,pix) dy_n[k][pix] * x_n[tap j at pix] M = Ks, red = N*P*Q
//
// Columns are the flattened index n*P*Q + pix in tiles of 128; tiles, main loop, LDS images
// and the weight-gradient split are those of gemm_kernels.h.
#pragma once
#include "conv_common.h"
#include "gemm_kernels.h"
#include "gemm_bf16_kernels.h"

namespace cs {

struct PmGeo {
  int Hp, Wp;   // extents of the image the taps are read from: x itself, or its zero-bordered copy
  int NPQ;      // N*P*Q columns
  int CT;       // column tiles of 128 (forward, input gradient)
  int NC;       // reduction chunks of 32 pixels per image (weight gradient)
};

// 4-byte LDS-DMA load: lane l's dword lands at lds_uniform + 4*l; address = uniform base + lane offset.
__device__ __forceinline__ void dma4_uv(const char* base_uniform, unsigned& lane_off, float* lds_uniform) {
  asm volatile("" : "+v"(lane_off));
  __builtin_amdgcn_global_load_lds(CS_GPTR(base_uniform + lane_off), CS_LPTR(lds_uniform), 4, 0, 0);
}

static __device__ __forceinline__ int pick8(const i32x4 (&v)[2], int r) { return v[r >> 2][r & 3]; }   // r: compile-time 0..7

// xb[n][c][hp][wp] = x[n][c][hp-ph][wp-pw] inside the image, 0 outside; converted to fp32.
template <typename Tin>
__global__ __launch_bounds__(256) void pm_border_copy_kernel(Geo g, int Hp, int Wp, const Tin* __restrict__ x,
                                                             float* __restrict__ xb) {
  const int64_t total = (int64_t)g.N * g.C * Hp * Wp;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int wp = (int)(i % Wp);
    const int64_t t = i / Wp;
    const int hp = (int)(t % Hp);
    const int64_t nc = t / Hp;
    const int h = hp - g.ph, v = wp - g.pw;
    float val = 0.f;
    if (h >= 0 && h < g.H && v >= 0 && v < g.W) val = load_as_f32<Tin>(x + (nc * g.H + h) * g.W + v);
    xb[i] = val;
  }
}

// dst[n][k][pix] (fp32, Ks channels) = src[n][k0+k][pix] (bf16, K channels).
__global__ __launch_bounds__(256) void pm_slice_to_f32_kernel(const uint16_t* __restrict__ src, int64_t srcImg,
                                                              int64_t dstImg, int N, float* __restrict__ dst) {
  const int64_t total = (int64_t)N * dstImg;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t n = i / dstImg;
    dst[i] = bf16_to_f32(src[n * srcImg + (i - n * dstImg)]);
  }
}

// tab[j] = byte offset of tap j = (c,r,s) from a window's origin inside one image of xb; entries
// past C*R*S repeat tap 0 (the filter operand is zero there).
__global__ void pm_tap_table_kernel(Geo g, int Hp, int Wp, int entries, int* __restrict__ tab) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= entries) return;
  const int j = i < g.CRS ? i : 0;
  const int c = j / g.RS, rs = j - c * g.RS;
  const int r = rs / g.S, s = rs - r * g.S;
  tab[i] = ((c * Hp + r) * Wp + s) * 4;
}

// The forward pass's two set-up jobs in one launch (they are a few microseconds each, most of it the launch):
// blocks below rblocks copy the filter rows to fp32 rows of pitch ldw, zero past C*R*S (repitch_rows_kernel's job),
// the others write the tap table (pm_tap_table_kernel's).
template <typename Tin>
__global__ __launch_bounds__(256) void pm_fwd_setup_kernel(Geo g, const Tin* __restrict__ wsrc, float* __restrict__ wdst,
                                                           int ldw, int rblocks, int Hp, int Wp, int entries,
                                                           int* __restrict__ tab) {
  if ((int)blockIdx.x >= rblocks) {
    const int i = ((int)blockIdx.x - rblocks) * blockDim.x + threadIdx.x;
    if (i >= entries) return;
    const int j = i < g.CRS ? i : 0;
    const int c = j / g.RS, rs = j - c * g.RS;
    const int r = rs / g.S, s = rs - r * g.S;
    tab[i] = ((c * Hp + r) * Wp + s) * 4;
    return;
  }
  const int64_t total = (int64_t)g.Ks * ldw;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)rblocks * blockDim.x) {
    const int r = (int)(i / ldw), c = (int)(i - (int64_t)r * ldw);
    wdst[i] = c < g.CRS ? load_as_f32<Tin>(wsrc + (int64_t)r * g.CRS + c) : 0.f;
  }
}

// Weight gradient: reduction chunk pc of an image covers 32 output pixels.  tab[pc*32 + kk] =
// byte offset of the window origin of that chunk's pixel kk inside one image of xb, or -1 if the
// pixel does not count.  The last chunk of an image is moved back so that it ends with the
// image's last pixel (the dy rows are read in place and must not be over-read); the pixels it
// shares with the chunk before are the ones that do not count.  Needs P*Q >= 32.
// The first workgroup also clears the zero page (zero_page may be null).
__global__ void pm_pixel_table_kernel(Geo g, int Wp, int NC, int* __restrict__ tab, float* __restrict__ zero_page) {
  if (zero_page && blockIdx.x == 0)
    for (int z = threadIdx.x; z < ZERO_PAGE_FLOATS; z += blockDim.x) zero_page[z] = 0.f;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= NC * 32) return;
  const int pc = i >> 5, kk = i & 31;
  const int start = pc == NC - 1 ? g.PQ - 32 : pc * 32;
  const int pix = start + kk;
  const int p = pix / g.Q, q = pix - p * g.Q;
  tab[i] = pix >= pc * 32 ? (p * g.sh * Wp + q * g.sw) * 4 : -1;
}

// Stores this wavefront's accumulators: rows m0.. of `rows` valid rows, columns = flattened
// (image, pixel) index; element (m, n, pix) goes to out[n*imgPitch + m*PQ + pix].
template <int MI, typename TOUT>
__device__ __forceinline__ void pm_store_tile(TOUT* __restrict__ out, int rows, int64_t imgPitch, int PQ, int NPQ,
                                              int m0, int ct, const f32x16 (&acc)[MI][Shape<MI>::NJ]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int j = 0; j < Shape<MI>::NJ; ++j) {
    const int col = ct * BN + Shape<MI>::col0(wave) + j * 32 + (lane & 31);
    if (col >= NPQ) continue;
    const int n = col / PQ, pix = col - n * PQ;
    TOUT* base = out + (int64_t)n * imgPitch + pix;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + Shape<MI>::row0(wave) + i * 32 + acc_row(v, lane);
        if (m < rows) store_from_f32<TOUT>(base + (int64_t)m * PQ, acc[i][j][v]);
      }
  }
}

// ---------------------------------------------------------------- forward ----
// B[kk][col] = xb[n][tap kk at the column's pixel] (row image).  A lane is a pixel: its byte
// offset (image + window origin) never changes; the tap's offset is added to the uniform base.
// The tap table is read with scalar loads one chunk ahead.
struct PmFwdLoadB {
  static constexpr bool COL = false;
  const char* xb;
  const CS_CONST int* tab;
  i32x4 cur[2], nxt[2];   // tap offsets of rows 8*wv .. 8*wv+7 of the chunk being issued / the next one
  unsigned laneoff[2];    // the lane's pixel in the tile's columns 0..63 and 64..127
  __device__ PmFwdLoadB(const Geo& g, const PmGeo& pg, const float* xb_, const int* tab_, int ct, int ch0)
      : xb((const char*)xb_), tab((const CS_CONST int*)tab_) {
    const int l = threadIdx.x & 63;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int col = min(ct * BN + 64 * h + l, pg.NPQ - 1);   // columns past the end repeat the last one (never stored)
      const int n = col / g.PQ, pix = col - n * g.PQ;
      const int p = pix / g.Q, q = pix - p * g.Q;
      laneoff[h] = (unsigned)(((n * g.C * pg.Hp) + p * g.sh) * pg.Wp + q * g.sw) * 4u;
    }
    fetch(ch0);
  }
  __device__ __forceinline__ void fetch(int ch) {
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const CS_CONST i32x4* po = (const CS_CONST i32x4*)(tab + ch * BK + 8 * wv);
    nxt[0] = po[0];
    nxt[1] = po[1];
  }
  // The table runs three chunks past the end and repeats tap 0 there, so dummy chunks need no test.
  __device__ __forceinline__ void begin(int ch, bool) {
    cur[0] = nxt[0];
    cur[1] = nxt[1];
    fetch(ch + 1);
  }
  __device__ __forceinline__ void issue(int i, float* dst) {   // rows 2i, 2i+1 of the wavefront's eight
    const char* b0 = xb + (unsigned)pick8(cur, 2 * i);
    const char* b1 = xb + (unsigned)pick8(cur, 2 * i + 1);
    dma4_uv(b0, laneoff[0], dst);
    dma4_uv(b0, laneoff[1], dst + 64);
    dma4_uv(b1, laneoff[0], dst + 128);
    dma4_uv(b1, laneoff[1], dst + 192);
  }
  __device__ __forceinline__ void end() {}
  __device__ __forceinline__ void restart() { fetch(0); }   // the same pixels again, from the first tap
};

// A store whose address is a wave-uniform base plus a 32-bit per-lane byte offset: the row of the tile moves in
// scalar registers and the lane's offset (its pixel) is reused by every store of the tile.
template <typename T>
__device__ __forceinline__ void store_uv(const char* base_uniform, unsigned& lane_off, float v) {
  asm volatile("" : "+v"(lane_off));
  store_from_f32<T>((T*)(base_uniform + lane_off), v);
}

// The stream of tiles of one persistent workgroup: a run of the line of CT x MB tiles, row tiles fastest, so
// that consecutive tiles share their column tile (the B loader is only restarted and the lanes' output offsets
// are kept).  A = rows of a dense matrix (FwdLoadA), B = MakeB(ct), output element (m, n, pix) at
// out[n*imgPitch + m*PQ + pix].
template <int MI, typename TOUT, class LB, class MakeB>
struct PmTiles {
  const Geo& g;
  const PmGeo& pg;
  const float* a;
  int lda, rows;
  MakeB makeB;
  TOUT* out;
  int64_t imgPitch;
  int mOrigin, MB;
  int ld, end;        // line position of the tile being loaded, end of the run
  int ld_mb, ld_ct;   // its coordinates
  int st_mb, st_ct;   // coordinates of the oldest tile not stored
  bool sameb;
  int cache_ct;       // column tile the lane offsets below belong to
  unsigned soff[2];
  bool sok[2];
  __device__ __forceinline__ void start(int begin, int end_) {
    ld = begin - 1;
    end = end_;
    ld_ct = st_ct = begin / MB;
    st_mb = begin - ld_ct * MB;
    ld_mb = st_mb - 1;
    sameb = false;
    cache_ct = -1;
  }
  __device__ __forceinline__ bool advance() {
    if (ld + 1 >= end) return false;
    ++ld;
    ++ld_mb;
    sameb = ld_mb < MB;
    if (!sameb) {
      ld_mb = 0;
      ++ld_ct;
    }
    return true;
  }
  __device__ __forceinline__ bool same_b() const { return sameb; }
  __device__ __forceinline__ FwdLoadA<MI> make_a() const { return FwdLoadA<MI>(a, lda, mOrigin + ld_mb * Shape<MI>::ROWS, rows); }
  __device__ __forceinline__ LB make_b() const { return makeB(ld_ct); }
  __device__ __forceinline__ void store(const f32x16 (&acc)[MI][Shape<MI>::NJ]) {
    constexpr int NJ = Shape<MI>::NJ;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m0 = mOrigin + st_mb * Shape<MI>::ROWS;
    const int ct = st_ct;
    if (++st_mb == MB) {
      st_mb = 0;
      ++st_ct;
    }
    if (cache_ct != ct) {   // the lane's two pixels: their offset in `out`, half-wave row included
      cache_ct = ct;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int col = ct * BN + Shape<MI>::col0(wave) + j * 32 + (lane & 31);
        sok[j] = col < pg.NPQ;
        const int c = min(col, pg.NPQ - 1);
        const int n = c / g.PQ, pix = c - n * g.PQ;
        soff[j] = (unsigned)((n * imgPitch + pix + 4 * (lane >> 5) * g.PQ) * (int64_t)sizeof(TOUT));
      }
    }
    const int64_t rowBytes = (int64_t)g.PQ * sizeof(TOUT);
    const char* sb = (const char*)out + (int64_t)(m0 + Shape<MI>::row0(wave)) * rowBytes;
    if (m0 + Shape<MI>::ROWS <= rows && (ct + 1) * BN <= pg.NPQ) {   // whole tile inside: no per-element tests
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            store_uv<TOUT>(sb + (i * 32 + 8 * (v >> 2) + (v & 3)) * rowBytes, soff[j], acc[i][j][v]);
      return;
    }
    const int mlane = m0 + Shape<MI>::row0(wave) + 4 * (lane >> 5);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      if (!sok[j]) continue;
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = i * 32 + 8 * (v >> 2) + (v & 3);
          if (mlane + r < rows) store_from_f32<TOUT>((TOUT*)(sb + r * rowBytes + soff[j]), acc[i][j][v]);
        }
    }
  }
};

struct PmFwdMakeB {
  const Geo* g;
  const PmGeo* pg;
  const float* xb;
  const int* tab;
  __device__ __forceinline__ PmFwdLoadB operator()(int ct) const { return PmFwdLoadB(*g, *pg, xb, tab, ct, 0); }
};

// y[n][k0+m][pix] for rows mOrigin.. of the slice; w rows have pitch ldw (a multiple of BK, zero past C*R*S).
// Persistent workgroups (grid = a multiple of 8, at most the chip's workgroup slots), each with a run of tiles.
template <int MI, typename TOUT>
__global__ __launch_bounds__(NT, 2) void fwd_pm_gemm_kernel(Geo g, PmGeo pg, const float* __restrict__ w, int ldw,
                                                            const float* __restrict__ xb, const int* __restrict__ tab,
                                                            TOUT* __restrict__ y, int mOrigin, int MB, int nch) {
  extern __shared__ __align__(16) float smem[];
  PmTiles<MI, TOUT, PmFwdLoadB, PmFwdMakeB> tiles{g, pg, w, ldw, g.Ks, PmFwdMakeB{&g, &pg, xb, tab},
                                                   y + (int64_t)g.k0 * g.PQ, (int64_t)g.K * g.PQ, mOrigin, MB};
  int begin, end;
  stream_run(MB * pg.CT, begin, end);
  tiles.start(begin, end);
  gemm_stream<FwdLoadA<MI>, PmFwdLoadB>(tiles, nch, smem, (g.CRS - (nch - 1) * BK + 7) >> 3);
}

// --------------------------------------------------------- input gradient ----
// B[kk][col] = dy[n][k0 + kk][pix] (row image), read in place: a row is a kernel, a lane a
// pixel (VEC4: four consecutive pixels with one 16-byte load, which needs P*Q % 4 == 0).
// Reduction rows past the slice repeat its last kernel: the filter operand is zero there.
template <bool VEC4>
struct PmDyLoadB {
  static constexpr bool COL = false;
  const char* dy;        // uniform: channel k0 of image 0
  unsigned rowBytes;     // one kernel's map
  int lastRow;           // Ks - 1
  unsigned laneoff[2];   // VEC4: [0] only
  unsigned upmask;
  int wv8, r0;
  __device__ PmDyLoadB(const Geo& g, const PmGeo& pg, const float* dy_k0, int64_t imgPitch, int ct)
      : dy((const char*)dy_k0), rowBytes((unsigned)g.PQ * 4u), lastRow(g.Ks - 1) {
    const int l = threadIdx.x & 63;
    wv8 = 8 * __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    upmask = l >= 32 ? ~0u : 0u;
    asm volatile("" : "+v"(upmask));
    if (VEC4) {
      const int col = min(ct * BN + 4 * (l & 31), pg.NPQ - 4);
      const int n = col / g.PQ, pix = col - n * g.PQ;
      laneoff[0] = (unsigned)(n * imgPitch + pix) * 4u;
      laneoff[1] = 0;
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int col = min(ct * BN + 64 * h + l, pg.NPQ - 1);
        const int n = col / g.PQ, pix = col - n * g.PQ;
        laneoff[h] = (unsigned)(n * imgPitch + pix) * 4u;
      }
    }
  }
  __device__ __forceinline__ void begin(int ch, bool live) { r0 = (live ? ch : 0) * BK + wv8; }
  __device__ __forceinline__ void issue(int i, float* dst) {
    const unsigned ra = (unsigned)min(r0 + 2 * i, lastRow) * rowBytes;
    const unsigned rb = (unsigned)min(r0 + 2 * i + 1, lastRow) * rowBytes;
    if (VEC4) {   // lower half-wave: row 2i, upper half-wave: row 2i+1
      unsigned off = laneoff[0] + ra + ((rb - ra) & upmask);
      dma16_uv(dy, off, dst);
    } else {
      dma4_uv(dy + ra, laneoff[0], dst);
      dma4_uv(dy + ra, laneoff[1], dst + 64);
      dma4_uv(dy + rb, laneoff[0], dst + 128);
      dma4_uv(dy + rb, laneoff[1], dst + 192);
    }
  }
  __device__ __forceinline__ void end() {}
  __device__ __forceinline__ void restart() {}
};

template <bool VEC4>
struct PmDyMakeB {
  const Geo* g;
  const PmGeo* pg;
  const float* dy_k0;
  int64_t imgPitch;
  __device__ __forceinline__ PmDyLoadB<VEC4> operator()(int ct) const { return PmDyLoadB<VEC4>(*g, *pg, dy_k0, imgPitch, ct); }
};

// T[n][j][pix] = sum_k wt[j][k] * dy[n][k0+k][pix]; wt = the slice's filter matrix transposed, pitch Ksp.
// Persistent workgroups, each with a run of the line of tiles.
template <int MI, bool VEC4>
__global__ __launch_bounds__(NT, 2) void bwd_data_pm_gemm_kernel(Geo g, PmGeo pg, const float* __restrict__ wt, int Ksp,
                                                                 const float* __restrict__ dy_k0, int64_t imgPitch,
                                                                 float* __restrict__ T, int mOrigin, int MB, int nch) {
  extern __shared__ __align__(16) float smem[];
  PmTiles<MI, float, PmDyLoadB<VEC4>, PmDyMakeB<VEC4>> tiles{g, pg, wt, Ksp, g.CRS, PmDyMakeB<VEC4>{&g, &pg, dy_k0, imgPitch},
                                                             T, (int64_t)g.CRS * g.PQ, mOrigin, MB};
  int begin, end;
  stream_run(MB * pg.CT, begin, end);
  tiles.start(begin, end);
  gemm_stream<FwdLoadA<MI>, PmDyLoadB<VEC4>>(tiles, nch, smem, (g.Ks - (nch - 1) * BK + 7) >> 3);
}

// dx[n][c][h][v] (+)= sum over the taps (r,s) whose window position (p,q) lands on (h,v) of
// T[n][(c,r,s)][p*Q+q], in increasing (r,s) order.  One thread per group of SW = stride consecutive
// input columns (SW = 0: any stride, one column per thread): column j of every group takes the
// same taps s at consecutive q, so for each (r, s) a wavefront reads 64 consecutive elements of
// one T row (with one column per thread and stride 4 it read 16-element pieces of four rows and
// fetched 2.15 times the bytes of T; now 1.5 times).  Misses read a clamped element and add a
// selected zero (branch-free: several taps' loads in flight).
template <typename TOUT, bool ACC, int SW, bool UNROLLED>
__global__ __launch_bounds__(256) void col2im_pm_kernel(Geo g, const float* __restrict__ T, TOUT* __restrict__ dx) {
  constexpr int NV = SW > 0 ? SW : 1;
  const int sw = SW > 0 ? SW : g.sw;
  const int groups = (g.W + NV - 1) / NV;   // column groups per input row
  const int64_t total = (int64_t)g.N * g.C * g.H * groups;
  // the grid is a multiple of 8: workgroups that follow each other on one XCD take neighbouring stretches, so the
  // cache lines that two stretches share (T rows are not line-aligned) are fetched into one L2 only
  const int64_t lb = (int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  for (int64_t i = lb * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int vg = (int)(i % groups);
    const int64_t t = i / groups;
    const int h = (int)(t % g.H);
    const int64_t nc = t / g.H;               // n*C + c
    const float* Tc = T + nc * g.RS * g.PQ;   // T[n][(c,0,0)][0]
    float acc[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = 0.f;
    if constexpr (UNROLLED) {
      // At most three taps per axis reach an element (ceil(R/sh), ceil(S/sw) <= 3): all 9*NV loads are issued
      // before the first is used, taps that do not exist or miss read a clamped element and add a selected zero.
      float val[3][NV][3];
#pragma unroll
      for (int rr = 0; rr < 3; ++rr) {
        const int r = (h + g.ph) % g.sh + rr * g.sh;
        const int hr = h + g.ph - r;
        const int p = hr / g.sh;
        const bool rok = r < g.R && hr >= 0 && p < g.P;
        const float* Tr = Tc + (int64_t)min(r, g.R - 1) * g.S * g.PQ + (rok ? p : 0) * g.Q;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          const int v = vg * NV + j;
#pragma unroll
          for (int k = 0; k < 3; ++k) {
            const int sx = (v + g.pw) % sw + k * sw;
            const int vs = v + g.pw - sx;
            const int q = vs / sw;
            const bool ok = rok && sx < g.S && vs >= 0 && q < g.Q;
            const float tv = Tr[(int64_t)min(sx, g.S - 1) * g.PQ + (ok ? q : 0)];
            val[rr][j][k] = ok ? tv : 0.f;
          }
        }
      }
#pragma unroll
      for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int rr = 0; rr < 3; ++rr)
#pragma unroll
          for (int k = 0; k < 3; ++k) acc[j] += val[rr][j][k];
    } else {
      for (int r = (h + g.ph) % g.sh; r < g.R; r += g.sh) {
        const int hr = h + g.ph - r;
        const int p = hr / g.sh;
        const bool rok = hr >= 0 && p < g.P;
        const float* Tr = Tc + (int64_t)r * g.S * g.PQ + (rok ? p : 0) * g.Q;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
          const int v = vg * NV + j;   // columns past W: computed on clamped elements, never stored
#pragma unroll 3
          for (int s = (v + g.pw) % sw; s < g.S; s += sw) {
            const int vs = v + g.pw - s;
            const int q = vs / sw;
            const bool ok = rok && vs >= 0 && q < g.Q;
            const float tv = Tr[(int64_t)s * g.PQ + (ok ? q : 0)];
            acc[j] += ok ? tv : 0.f;
          }
        }
      }
    }
    TOUT* o = dx + ((nc * g.H + h) * (int64_t)g.W + vg * NV);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      if (vg * NV + j < g.W) {
        float a = acc[j];
        if (ACC) a += load_as_f32<TOUT>(o + j);
        store_from_f32<TOUT>(o + j, a);
      }
    }
  }
}

// ---------------------------------------------------------- weight gradient ----
// Reduction chunk = 32 pixels of one image; the chunks (n, pc) of a split are walked with
// uniform carry counters: step i of split z is chunk z + i*splits.
struct PmChunkWalk {
  int n, pc, NC, dn, dpc;
  __device__ PmChunkWalk(int first, int stride, int NC_) : n(first / NC_), pc(first - (first / NC_) * NC_), NC(NC_),
                                                           dn(stride / NC_), dpc(stride - (stride / NC_) * NC_) {}
  __device__ __forceinline__ void next() {
    pc += dpc;
    const int c = pc >= NC;
    pc -= c ? NC : 0;
    n += dn + c;
  }
};

// A[m][kk] = dy[n][k0+m0+m][start(pc) + kk] (col image), read in place.  VEC4 (P*Q % 4 == 0):
// 16-byte loads as in the other passes' filter operand; otherwise 4-byte loads, each lane
// fetching the element that the col image's swizzle puts at its LDS position.  Rows past the
// slice repeat its last kernel (never stored).
template <int MI_, bool VEC4>
struct PmDyLoadA {
  static constexpr bool COL = true;
  static constexpr int MI = MI_;
  const char* dy;        // uniform: channel k0 of image 0
  const char* ub;
  int64_t imgBytes;
  int PQ, N;
  unsigned off[VEC4 ? Shape<MI>::NLOAD : 4 * Shape<MI>::NLOAD];
  PmChunkWalk walk;
  __device__ PmDyLoadA(const Geo& g, const PmGeo& pg, const float* dy_k0, int64_t imgPitch, int m0, int first, int stride)
      : dy((const char*)dy_k0), imgBytes(imgPitch * 4), PQ(g.PQ), N(g.N), walk(first, stride, pg.NC) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (VEC4) {
#pragma unroll
      for (int i = 0; i < Shape<MI>::NLOAD; ++i) {
        const int kq4 = 4 * ((l & 7) ^ col_key(Shape<MI>::WROWS * wv + 8 * i + (l >> 3)));
        const int m = min(m0 + Shape<MI>::WROWS * wv + 8 * i + (l >> 3), g.Ks - 1);
        off[i] = ((unsigned)m * (unsigned)g.PQ + kq4) * 4u;
      }
    } else {
#pragma unroll
      for (int i = 0; i < Shape<MI>::NLOAD; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int row = Shape<MI>::WROWS * wv + 8 * i + 2 * jj + (l >> 5);   // row of the tile
          const int kk = ((((l & 31) >> 2) ^ col_key(row)) << 2) + (l & 3);   // element stored at this lane's LDS position
          const int m = min(m0 + row, g.Ks - 1);
          off[i * 4 + jj] = ((unsigned)m * (unsigned)g.PQ + kk) * 4u;
        }
    }
  }
  __device__ __forceinline__ void begin(int, bool live) {   // dummy chunks re-read the first chunk of image 0
    const int n = live ? walk.n : 0, pc = live ? walk.pc : 0;
    const int start = pc == walk.NC - 1 ? PQ - 32 : pc * 32;
    ub = dy + ((int64_t)n * imgBytes + (int64_t)start * 4);
  }
  __device__ __forceinline__ void issue(int i, float* dst) {
    if (VEC4) {
      dma16_uv(ub, off[i], dst);
    } else {
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) dma4_uv(ub, off[i * 4 + jj], dst + 64 * jj);
    }
  }
  __device__ __forceinline__ void end() { walk.next(); }
};

// B[kk][j] = xb[n][tap j at pixel kk of the chunk] (row image): a row is a pixel (uniform base from
// the pixel table, scalar loads one chunk ahead), a lane is a tap with a constant offset.  Pixels
// that do not count (table entry -1) read the zero page.  Taps past C*R*S repeat tap 0 (never stored).
struct PmTapLoadB {
  static constexpr bool COL = false;
  const char* xb;
  const char* zero;
  const char* img;       // uniform: image of the chunk being issued
  const CS_CONST int* pixtab;
  int64_t imgBytes;
  int N;
  i32x4 cur[2], nxt[2];
  unsigned tapoff[2], zoff;
  PmChunkWalk walk;
  __device__ PmTapLoadB(const Geo& g, const PmGeo& pg, const float* xb_, const float* zero_, const int* pixtab_, int j0,
                        int first, int stride)
      : xb((const char*)xb_), zero((const char*)zero_), pixtab((const CS_CONST int*)pixtab_),
        imgBytes((int64_t)g.C * pg.Hp * pg.Wp * 4), N(g.N), walk(first, stride, pg.NC) {
    const int l = threadIdx.x & 63;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int j = j0 + 64 * h + l;
      const int jj = j < g.CRS ? j : 0;
      const int c = jj / g.RS, rs = jj - c * g.RS;
      const int r = rs / g.S, s = rs - r * g.S;
      tapoff[h] = (unsigned)((c * pg.Hp + r) * pg.Wp + s) * 4u;
    }
    zoff = (unsigned)l * 4u;
    fetch(walk.pc);
  }
  __device__ __forceinline__ void fetch(int pc) {
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const CS_CONST i32x4* po = (const CS_CONST i32x4*)(pixtab + pc * 32 + 8 * wv);
    nxt[0] = po[0];
    nxt[1] = po[1];
  }
  __device__ __forceinline__ void begin(int, bool) {   // dummy chunks read real pixels of the last image
    cur[0] = nxt[0];
    cur[1] = nxt[1];
    img = xb + (int64_t)min(walk.n, N - 1) * imgBytes;
  }
  __device__ __forceinline__ void issue(int i, float* dst) {
#pragma unroll
    for (int rr = 0; rr < 2; ++rr) {
      const int po = pick8(cur, 2 * i + rr);
      const bool live = po >= 0;
      const char* b = live ? img + (unsigned)po : zero;
      unsigned o0 = live ? tapoff[0] : zoff, o1 = live ? tapoff[1] : zoff;
      dma4_uv(b, o0, dst + 128 * rr);
      dma4_uv(b, o1, dst + 128 * rr + 64);
    }
  }
  __device__ __forceinline__ void end() {
    walk.next();
    fetch(walk.pc);
  }
};

// out[z][m][j]: split z of the weight gradient (chunks z, z + splits, ...); tiles * splits work
// items dealt to the XCDs in contiguous blocks, as in bwd_weight_gemm_kernel.
template <int MI, bool VEC4>
__global__ __launch_bounds__(NT) void bwd_weight_pm_gemm_kernel(Geo g, PmGeo pg, const float* __restrict__ dy_k0,
                                                                int64_t imgPitch, const float* __restrict__ xb,
                                                                const float* __restrict__ zero,
                                                                const int* __restrict__ pixtab,
                                                                float* __restrict__ out, int64_t splitStride,
                                                                int mOrigin, int rowBase, int MB, int CT, int nch,
                                                                int splits) {
  extern __shared__ __align__(16) float smem[];
  const int tiles = MB * CT;
  int item;
  if (!line_contiguous(blockIdx.x, tiles * splits, item)) return;
  const int z = item / tiles, L = item - z * tiles;
  int mb, ct;
  tile_from_line(L, MB, CT, mb, ct);
  const int m0 = mOrigin + mb * Shape<MI>::ROWS;
  const int count = (nch - z + splits - 1) / splits;
  f32x16 acc[Shape<MI>::RB][Shape<MI>::NJ];
#pragma unroll
  for (int i = 0; i < Shape<MI>::RB; ++i)
#pragma unroll
    for (int j = 0; j < Shape<MI>::NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  PmDyLoadA<MI, VEC4> la(g, pg, dy_k0, imgPitch, m0, z, splits);
  PmTapLoadB lb(g, pg, xb, zero, pixtab, ct * BN, z, splits);
  gemm_mainloop(la, lb, 0, count, smem, acc);
  bwd_weight_store_tile<MI>(g, out + (int64_t)z * splitStride, m0, rowBase, ct, acc);
}

// ------------------------------------------- forward, bf16 matrix cores ----
// Few input channels in bfloat16.  v_mfma_f32_32x32x16_bf16 wants eight consecutive reduction
// elements per lane, which a gather of single taps cannot give; one filter ROW can: in a copy of x
// with the channels innermost, xc[n][hb][wb][Cp] (Cp = 4, 8 or 16 channels, zero filled; Cp = 4 only with an even
// horizontal stride, so that every window starts on a 16-byte boundary; zero border
// of ph rows / pw columns, and enough columns on the right that every read below stays inside),
// the taps (r, s..s+WPC-1, all channels) of a window are 64 consecutive elements.  So the
// reduction is laid out as (r, j, 64 elements): R * CPR chunks with CPR = ceil(S / WPC),
// WPC = 64 / Cp window columns per chunk, and the filters are re-laid to match,
// wk[k][r][CPR * WPC][Cp], zero where s >= S or c >= C: the columns a chunk reads past the window
// meet zero weights.  A column of the GEMM is an output pixel of one image; its byte offset in xc
// never changes, the chunk's (r, j) offset moves in the uniform base: the addressing of the other
// bf16 kernels.  Tiles are 128 kernels x 128 pixels, y is written in place (bf16, NCHW).
struct Pm16Geo {
  int Cp, WPC, CPR, Hb, Wb;   // padded channels, window columns per chunk, chunks per filter row, extents of xc
};

// xc[n][hb][wb][c] = x[n][c][hb-ph][wb-pw] inside the image and for c < C, else 0.  One thread per (n, hb, wb).
template <int CP>
__global__ __launch_bounds__(256) void pm16_channels_last_kernel(Geo g, Pm16Geo pg, const uint16_t* __restrict__ x,
                                                                 uint16_t* __restrict__ xc) {
  const int64_t total = (int64_t)g.N * pg.Hb * pg.Wb;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int wb = (int)(i % pg.Wb);
    const int64_t t = i / pg.Wb;
    const int hb = (int)(t % pg.Hb);
    const int64_t n = t / pg.Hb;
    const int h = hb - g.ph, v = wb - g.pw;
    const bool in = h >= 0 && h < g.H && v >= 0 && v < g.W;
    const uint16_t* src = x + (n * g.C * g.H + (in ? h : 0)) * (int64_t)g.W + (in ? v : 0);
    uint16_t vals[CP];
#pragma unroll
    for (int c = 0; c < CP; ++c) vals[c] = (in && c < g.C) ? src[(int64_t)min(c, g.C - 1) * g.HW] : (uint16_t)0;
    if constexpr (CP == 4) {
      uint2 u;
      u.x = vals[0] | ((unsigned)vals[1] << 16);
      u.y = vals[2] | ((unsigned)vals[3] << 16);
      *(uint2*)(xc + i * CP) = u;
    }
    uint4* dst = (uint4*)(xc + i * CP);
#pragma unroll
    for (int q = 0; q < CP / 8; ++q) {
      uint4 u;
      u.x = vals[8 * q + 0] | ((unsigned)vals[8 * q + 1] << 16);
      u.y = vals[8 * q + 2] | ((unsigned)vals[8 * q + 3] << 16);
      u.z = vals[8 * q + 4] | ((unsigned)vals[8 * q + 5] << 16);
      u.w = vals[8 * q + 6] | ((unsigned)vals[8 * q + 7] << 16);
      dst[q] = u;
    }
  }
}

// wk[k][r][s'][c'] = w[k0+k][c'][r][s'] for s' < S, c' < C, else 0; one thread per element of wk.
__global__ __launch_bounds__(256) void pm16_filters_kernel(Geo g, Pm16Geo pg, const uint16_t* __restrict__ w_k0,
                                                           uint16_t* __restrict__ wk) {
  const int SP = pg.CPR * pg.WPC;
  const int64_t total = (int64_t)g.Ks * g.R * SP * pg.Cp;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(i % pg.Cp);
    int64_t t = i / pg.Cp;
    const int s = (int)(t % SP);
    t /= SP;
    const int r = (int)(t % g.R);
    const int64_t k = t / g.R;
    wk[i] = (c < g.C && s < g.S) ? w_k0[((k * g.C + c) * g.R + r) * g.S + s] : (uint16_t)0;
  }
}

// B^T[col][kk] = xc[n][p*sh + r][q*sw + j*WPC ..][..]: 64 consecutive elements per column and chunk.
struct Pm16LoadB {
  const char* xc;     // uniform
  const char* ub;
  unsigned off[4];
  unsigned rowBytes;  // one row of xc
  int CPR;
  int r, j;           // uniform walk over the next chunk to issue
  __device__ Pm16LoadB(const Geo& g, const Pm16Geo& pg, const uint16_t* xc_, int NPQ, int ct, int ch0)
      : xc((const char*)xc_), rowBytes((unsigned)pg.Wb * (unsigned)pg.Cp * 2u), CPR(pg.CPR) {
    const int l = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int col = min(ct * BN + wv * 32 + 8 * i + (l >> 3), NPQ - 1);   // columns past the end: computed, never stored
      const int n = col / g.PQ, pix = col - n * g.PQ;
      const int pp = pix / g.Q, q = pix - pp * g.Q;
      off[i] = (unsigned)((((int64_t)n * pg.Hb + pp * g.sh) * pg.Wb + q * g.sw) * pg.Cp + slot8(l, i)) * 2u;
    }
    r = ch0 / CPR;
    j = ch0 - r * CPR;
  }
  __device__ __forceinline__ void begin(int, bool live) {
    ub = xc + (live ? (unsigned)r * rowBytes + (unsigned)j * (BK16 * 2u) : 0u);
  }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {   // branch-free carry over (j, r)
    ++j;
    const int c = j == CPR;
    j = c ? 0 : j;
    r += c;
  }
};

// grid = grid_contiguous(MB * CT): one workgroup per tile, tiles dealt to the XCDs in contiguous blocks.
__global__ __launch_bounds__(NT) void fwd16_pm_gemm_kernel(Geo g, Pm16Geo pg, const bf16_t* __restrict__ wk, int64_t ldw,
                                                           const bf16_t* __restrict__ xc, uint16_t* __restrict__ y,
                                                           int NPQ, int MB, int CT, int nch) {
  extern __shared__ __align__(16) float smem[];
  int L;
  if (!line_contiguous(blockIdx.x, MB * CT, L)) return;
  int mb, ct;
  tile_from_line(L, MB, CT, mb, ct);
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][jj][v] = 0.f;
  Fwd16LoadA la(wk, ldw, mb * BM, g.Ks);
  Pm16LoadB lb(g, pg, xc, NPQ, ct, 0);
  gemm16_mainloop(la, lb, 0, nch, smem, acc);
  pm_store_tile<2, uint16_t>(y + (int64_t)g.k0 * g.PQ, g.Ks, (int64_t)g.K * g.PQ, g.PQ, NPQ, mb * BM, ct, acc);
}

// ------------------------------------ input gradient, bf16 matrix cores ----
// T = w^T dy is a 1 x 1 convolution of dy with C*R*S "kernels" over the slice's Ks "channels": with the
// maps of the slice copied channels-last, dyc[(n, pix)][Kp] (Kp = Ks rounded up to the chunk, zero
// filled), the 64 reduction elements of a column and chunk are consecutive, and the filters transposed,
// wt[(c,r,s)][Kp].  B^T[col][kk] = dyc[col][ch*64 + kk].
struct Pm16DyLoadB {
  const char* dyc;   // uniform
  const char* ub;
  unsigned off[4];
  __device__ Pm16DyLoadB(const uint16_t* dyc_, int Kp, int NPQ, int ct) : dyc((const char*)dyc_) {
    const int l = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int col = min(ct * BN + wv * 32 + 8 * i + (l >> 3), NPQ - 1);   // columns past the end: computed, never stored
      off[i] = ((unsigned)col * (unsigned)Kp + slot8(l, i)) * 2u;
    }
  }
  __device__ __forceinline__ void begin(int ch, bool live) { ub = dyc + (live ? (unsigned)ch * (BK16 * 2u) : 0u); }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {}
};

// T[n][j][pix] = sum_k wt[j][k] * dyc[(n, pix)][k], fp32 (a bf16 T would halve this pass's traffic, but sums of
// taps that cancel then miss the bf16 tolerance); one workgroup per 128 x 128 tile, tiles dealt to the
// XCDs in contiguous blocks (grid = grid_contiguous(MB * CT)).
__global__ __launch_bounds__(NT) void bwd_data16_pm_gemm_kernel(const bf16_t* __restrict__ wt, int Kp, int CRS,
                                                                const bf16_t* __restrict__ dyc, float* __restrict__ T,
                                                                int PQ, int NPQ, int MB, int CT) {
  extern __shared__ __align__(16) float smem[];
  int L;
  if (!line_contiguous(blockIdx.x, MB * CT, L)) return;
  int mb, ct;
  tile_from_line(L, MB, CT, mb, ct);
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][jj][v] = 0.f;
  Fwd16LoadA la(wt, Kp, mb * BM, CRS);
  Pm16DyLoadB lb(dyc, Kp, NPQ, ct);
  gemm16_mainloop(la, lb, 0, Kp / BK16, smem, acc);
  pm_store_tile<2, float>(T, CRS, (int64_t)CRS * PQ, PQ, NPQ, mb * BM, ct, acc);
}

}  // namespace cs
