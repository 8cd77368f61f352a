// The three matrix-core passes.  Each is an implicit GEMM on 128x128 tiles whose
// 32-lane column blocks are "32 images at one pixel" (fwd, bwd_data) or 32 filter
// taps (bwd_weight); the operand loaders below are the only pass-specific code.
// A loader computes, per lane, the global address of the 16 bytes that lane moves
// into LDS for each of its wavefront's four DMA loads per chunk (see the staging
// notes in conv_common.h for the row and col tile images).
#pragma once
#include "conv_common.h"

namespace cs {

// Wave-uniform LDS destination of DMA load number i of wavefront wv.
__device__ __forceinline__ float* dma_dst(float* tile, int wv, int i) { return tile + (wv * 4 + i) * 256; }

// ---------------------------------------------------------------- forward ----
// A[m][kk] = w[k0+m0+m][kk]: rows of the (re-pitched) filter matrix, col image.
struct FwdLoadA {
  static constexpr bool COL = true;
  const float* p[4];
  const float* zero;
  int kq4, cols;  // float offset of this lane's slot inside a chunk; valid row length
  __device__ FwdLoadA(const float* w, int ldw, int cols_, int m0, int Ks, const float* zero_)
      : zero(zero_), cols(cols_) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    kq4 = 4 * ((l & 7) ^ (l >> 3));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = min(m0 + 32 * wv + 8 * i + (l >> 3), Ks - 1);  // rows past the slice repeat the last one
      p[i] = w + (int64_t)m * ldw + kq4;
    }
  }
  __device__ __forceinline__ void issue(int ch, float* tile, int wv) {
    const bool kok = ch * BK + kq4 < cols;
#pragma unroll
    for (int i = 0; i < 4; ++i) dma16(kok ? p[i] + ch * BK : zero, dma_dst(tile, wv, i));
  }
};

// B[kk][col] = x_t[tap kk of the column block's pixel][n] (row image), zero where the
// tap falls into the padding.  Each lane walks its four reduction rows kk = (c,r,s)
// with carry arithmetic (+32 per chunk), so no division or table sits in the loop.
struct FwdLoadB {
  static constexpr bool COL = false;
  const float* xt;
  const float* zero;
  int base, h0, w0, H, W, C, R, S, HW, Np;
  int dc, dr, ds;         // (c,r,s) increments of one chunk
  int cc[4], rr[4], ss[4];
  bool cbok;
  __device__ FwdLoadB(const Geo& g, const float* xt_, int ct, const float* zero_) : xt(xt_), zero(zero_) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int cq = l & 31;
    const int gcb = ct * 4 + (cq >> 3);
    cbok = gcb < g.PQ * g.NB;
    const int pix = cbok ? gcb / g.NB : 0;
    const int nb = cbok ? gcb - pix * g.NB : 0;
    const int p = pix / g.Q, q = pix - p * g.Q;
    h0 = p * g.sh - g.ph;
    w0 = q * g.sw - g.pw;
    H = g.H; W = g.W; C = g.C; R = g.R; S = g.S; HW = g.HW; Np = g.Np;
    base = nb * 32 + 4 * (cq & 7);
    dc = BK / g.RS;
    const int rem = BK - dc * g.RS;
    dr = rem / g.S;
    ds = rem - dr * g.S;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int kk = 8 * wv + 2 * i + (l >> 5);
      cc[i] = kk / g.RS;
      const int rs = kk - cc[i] * g.RS;
      rr[i] = rs / g.S;
      ss[i] = rs - rr[i] * g.S;
    }
  }
  __device__ __forceinline__ void issue(int, float* tile, int wv) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int hh = h0 + rr[i], vv = w0 + ss[i];
      const bool ok = cbok && cc[i] < C && (unsigned)hh < (unsigned)H && (unsigned)vv < (unsigned)W;
      dma16(ok ? xt + ((cc[i] * HW + hh * W + vv) * Np + base) : zero, dma_dst(tile, wv, i));
      // advance (c,r,s) by one chunk
      ss[i] += ds;
      if (ss[i] >= S) { ss[i] -= S; rr[i] += 1; }
      rr[i] += dr;
      if (rr[i] >= R) { rr[i] -= R; cc[i] += 1; }
      cc[i] += dc;
    }
  }
};

// y_t[k][pix][n] for the slice; one workgroup per 128 kernels x 4 column blocks.
__global__ __launch_bounds__(NT) void fwd_gemm_kernel(Geo g, const float* __restrict__ w, int ldw,
                                                      int wcols, const float* __restrict__ xt,
                                                      const float* __restrict__ zero,
                                                      float* __restrict__ yt, int MB, int CT, int nch) {
  extern __shared__ __align__(16) float smem[];
  int mb, ct;
  if (!tile_contiguous(blockIdx.x, MB, CT, mb, ct)) return;
  const int m0 = mb * BM;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  FwdLoadA la(w, ldw, wcols, m0, g.Ks, zero);
  FwdLoadB lb(g, xt, ct, zero);
  gemm_mainloop(la, lb, 0, nch, smem, acc);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int gcb = ct * 4 + wn * 2 + j;
    if (gcb >= g.PQ * g.NB) continue;
    const int pix = gcb / g.NB, nb = gcb - pix * g.NB;
    const int n = nb * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 64 + i * 32 + acc_row(v, lane);
        if (m < g.Ks) yt[((int64_t)m * g.PQ + pix) * g.Np + n] = acc[i][j][v];
      }
  }
}

// --------------------------------------------------------- input gradient ----
// Reduction runs over (tap, k): only taps that reach the tile's pixels, k inner.
// A^T[k][c] = w_t[tap][k][c] (filters re-laid with c innermost, pitch Cp), row image.
struct BwdDataLoadA {
  static constexpr bool COL = false;
  const float* wt;
  const float* zero;
  const int* taps;
  int Ks, Cp, S, nkc, c, krow, ti, kc;
  int64_t tapbase;
  __device__ BwdDataLoadA(const Geo& g, const float* wt_, int Cp_, int m0, const int* taps_, int nkc_,
                          const float* zero_)
      : wt(wt_), zero(zero_), taps(taps_), Ks(g.Ks), Cp(Cp_), S(g.S), nkc(nkc_), ti(0), kc(0), tapbase(0) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    c = m0 + 4 * (l & 31);
    krow = 8 * wv + (l >> 5);
  }
  __device__ __forceinline__ void issue(int, float* tile, int wv) {
    if (kc == 0) {
      const int e = taps[ti];
      tapbase = (int64_t)((e >> 16) * S + (e & 0xffff)) * Ks * Cp;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = kc * BK + krow + 2 * i;
      const bool ok = k < Ks && c < Cp;
      dma16(ok ? wt + (tapbase + (int64_t)k * Cp + c) : zero, dma_dst(tile, wv, i));
    }
    if (++kc == nkc) {
      kc = 0;
      ++ti;
    }
  }
};

// B[k][col] = dy_t[k][p][q][n] (row image) with (p,q) the output pixel whose window
// puts the current tap on the column block's input pixel; zero if there is none.
struct BwdDataLoadB {
  static constexpr bool COL = false;
  const float* dyt;
  const float* zero;
  const int* taps;
  int Ks, nkc, krow, ti, kc;
  int hp, vp, sh, sw, P, Q, PQNp, nboff, Np;  // hp = h + pad_h, vp = v + pad_w of this lane's pixel
  int off;
  bool cbok, tapok;
  __device__ BwdDataLoadB(const Geo& g, const float* dyt_, const int* perm, int ct, const int* taps_, int nkc_,
                          const float* zero_)
      : dyt(dyt_), zero(zero_), taps(taps_), Ks(g.Ks), nkc(nkc_), ti(0), kc(0), off(0), tapok(false) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int cq = l & 31;
    const int gcb = ct * 4 + (cq >> 3);
    cbok = gcb < g.HW * g.NB;
    const int sp = cbok ? gcb / g.NB : 0;
    const int nb = cbok ? gcb - sp * g.NB : 0;
    const int px = perm[sp];
    hp = px / g.W + g.ph;
    vp = px % g.W + g.pw;
    sh = g.sh; sw = g.sw; P = g.P; Q = g.Q; Np = g.Np;
    PQNp = g.PQ * g.Np;
    nboff = nb * 32 + 4 * (cq & 7);
    krow = 8 * wv + (l >> 5);
  }
  __device__ __forceinline__ void issue(int, float* tile, int wv) {
    if (kc == 0) {
      const int e = taps[ti];
      const int hr = hp - (e >> 16), vs = vp - (e & 0xffff);
      const int p = hr / sh, q = vs / sw;
      tapok = cbok && hr >= 0 && vs >= 0 && p * sh == hr && q * sw == vs && p < P && q < Q;
      off = (p * Q + q) * Np + nboff;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = kc * BK + krow + 2 * i;
      const bool ok = tapok && k < Ks;
      dma16(ok ? dyt + ((int64_t)k * PQNp + off) : zero, dma_dst(tile, wv, i));
    }
    if (++kc == nkc) {
      kc = 0;
      ++ti;
    }
  }
};

// dx_t[c][pixel][n]; column tiles follow the pixel order in perm (heaviest first).
__global__ __launch_bounds__(NT) void bwd_data_gemm_kernel(Geo g, const float* __restrict__ wt, int Cp,
                                                           const float* __restrict__ dyt,
                                                           const int* __restrict__ perm,
                                                           const float* __restrict__ zero,
                                                           float* __restrict__ dxt, int MB, int CT) {
  extern __shared__ __align__(16) float smem[];
  __shared__ int s_taps[1024];
  __shared__ int s_ntaps;
  int mb, ct;
  if (!tile_dealt(blockIdx.x, MB, CT, mb, ct)) return;
  const int m0 = mb * BM;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // Taps that reach at least one of the tile's (up to four) pixels, in (r,s) order.
  if (wave == 0) {
    int hp[4], vp[4];
    bool ok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gcb = ct * 4 + j;
      ok[j] = gcb < g.HW * g.NB;
      const int px = perm[ok[j] ? gcb / g.NB : 0];
      hp[j] = px / g.W + g.ph;
      vp[j] = px % g.W + g.pw;
    }
    int cnt = 0;
    for (int b = 0; b < g.RS; b += 64) {
      const int tp = b + lane;
      const int rr = tp / g.S, ss = tp - rr * g.S;
      bool any = false;
      if (tp < g.RS) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int hr = hp[j] - rr, vs = vp[j] - ss;
          any |= ok[j] && hr >= 0 && vs >= 0 && hr % g.sh == 0 && vs % g.sw == 0 &&
                 hr / g.sh < g.P && vs / g.sw < g.Q;
        }
      }
      const unsigned long long mask = __ballot(any);
      if (any) s_taps[cnt + __popcll(mask & ((1ull << lane) - 1ull))] = (rr << 16) | ss;
      cnt += __popcll(mask);
    }
    if (lane == 0) s_ntaps = cnt;
  }
  __syncthreads();
  const int ntaps = s_ntaps;
  const int nkc = (g.Ks + BK - 1) / BK;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  BwdDataLoadA la(g, wt, Cp, m0, s_taps, nkc, zero);
  BwdDataLoadB lb(g, dyt, perm, ct, s_taps, nkc, zero);
  gemm_mainloop(la, lb, 0, ntaps * nkc, smem, acc);

  const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int gcb = ct * 4 + wn * 2 + j;
    if (gcb >= g.HW * g.NB) continue;
    const int sp = gcb / g.NB, nb = gcb - sp * g.NB;
    const int px = perm[sp];
    const int n = nb * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int c = m0 + wm * 64 + i * 32 + acc_row(v, lane);
        if (c < g.C) dxt[((int64_t)c * g.HW + px) * g.Np + n] = acc[i][j][v];
      }
  }
}

// -------------------------------------------------------- weight gradient ----
// Reduction runs over (pixel, n) in chunks of 32 images of one output pixel.
// A[m][kk] = dy_t[m0+m][pix][n]: dense rows, col image.
struct BwdWeightLoadA {
  static constexpr bool COL = true;
  const float* p[4];
  __device__ BwdWeightLoadA(const Geo& g, const float* dyt, int m0) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int kq4 = 4 * ((l & 7) ^ (l >> 3));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = min(m0 + 32 * wv + 8 * i + (l >> 3), g.Ks - 1);  // rows past the slice repeat the last one
      p[i] = dyt + (int64_t)m * g.PQ * g.Np + kq4;
    }
  }
  __device__ __forceinline__ void issue(int ch, float* tile, int wv) {
#pragma unroll
    for (int i = 0; i < 4; ++i) dma16(p[i] + (int64_t)ch * BK, dma_dst(tile, wv, i));
  }
};

// B^T[j][kk] = x_t[c_j][p*sh-ph+r_j][q*sw-pw+s_j][n] (col image); zero where tap j is in
// the padding or j is past C*R*S.
struct BwdWeightLoadB {
  static constexpr bool COL = true;
  const float* xt;
  const float* zero;
  int colbase[4], rj[4], sj[4];
  bool colok[4];
  int NB, Q, sh, sw, ph, pw, H, W, Np, kq4;
  __device__ BwdWeightLoadB(const Geo& g, const float* xt_, int j0, const float* zero_) : xt(xt_), zero(zero_) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    NB = g.NB; Q = g.Q; sh = g.sh; sw = g.sw; ph = g.ph; pw = g.pw; H = g.H; W = g.W; Np = g.Np;
    kq4 = 4 * ((l & 7) ^ (l >> 3));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = j0 + 32 * wv + 8 * i + (l >> 3);
      colok[i] = j < g.CRS;
      const int jj = colok[i] ? j : 0;
      const int c = jj / g.RS, rs = jj - c * g.RS;
      rj[i] = rs / g.S;
      sj[i] = rs - rj[i] * g.S;
      colbase[i] = c * g.HW * g.Np;
    }
  }
  __device__ __forceinline__ void issue(int ch, float* tile, int wv) {
    const int pix = ch / NB, nb = ch - pix * NB;
    const int p = pix / Q, q = pix - p * Q;
    const int h0 = p * sh - ph, v0 = q * sw - pw;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int hh = h0 + rj[i], vv = v0 + sj[i];
      const bool ok = colok[i] && (unsigned)hh < (unsigned)H && (unsigned)vv < (unsigned)W;
      dma16(ok ? xt + (colbase[i] + (hh * W + vv) * Np + nb * 32 + kq4) : zero, dma_dst(tile, wv, i));
    }
  }
};

// out[z][m][j] partial (or final when one split) weight gradients of the slice.
__global__ __launch_bounds__(NT) void bwd_weight_gemm_kernel(Geo g, const float* __restrict__ dyt,
                                                             const float* __restrict__ xt,
                                                             const float* __restrict__ zero,
                                                             float* __restrict__ out, int64_t splitStride,
                                                             int MB, int CT, int nch, int chPerSplit) {
  extern __shared__ __align__(16) float smem[];
  int mb, ct;
  if (!tile_contiguous(blockIdx.x, MB, CT, mb, ct)) return;
  const int m0 = mb * BM, j0 = ct * BN;
  const int z = blockIdx.y;
  const int ch0 = z * chPerSplit;
  const int ch1 = min(nch, ch0 + chPerSplit);
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  BwdWeightLoadA la(g, dyt, m0);
  BwdWeightLoadB lb(g, xt, j0, zero);
  gemm_mainloop(la, lb, ch0, ch1, smem, acc);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  float* o = out + (int64_t)z * splitStride;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = j0 + wn * 64 + j * 32 + (lane & 31);
    if (col >= g.CRS) continue;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 64 + i * 32 + acc_row(v, lane);
        if (m < g.Ks) o[(int64_t)m * g.CRS + col] = acc[i][j][v];
      }
  }
}

}  // namespace cs
