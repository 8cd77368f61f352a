// The three matrix-core passes.  Each is an implicit GEMM on 128x128 tiles whose
// 32-lane column blocks are "32 images at one pixel" (fwd, bwd_data) or 32 filter
// taps (bwd_weight); the operand loaders below are the only pass-specific code.
#pragma once
#include "conv_common.h"

namespace cs {

// Thread -> element maps used by the loaders (256 threads, 4 float4 each):
//   "row" map : 32 reduction rows x 32 float4 columns; thread covers rows t/32 + 8i.
//   "col" map : 128 tile rows x 8 float4 along the reduction; thread covers rows t/8 + 32i
//               and stores transposed into LDS.

// ---------------------------------------------------------------- forward ----
// A[m][kk] = w[k0+m0+m][kk], rows of the (re-pitched) filter matrix.
struct FwdLoadA {
  static constexpr int LD = LDT;
  const float* base[4];
  bool rowok[4];
  int kq, cols;  // float offset of this thread's quad inside a chunk; valid row length
  f32x4 r[4];
  bool okv[4];  // value mask, applied when the registers go to LDS
  __device__ FwdLoadA(const float* w, int ldw, int cols_, int m0, int Ks) {
    const int t = threadIdx.x;
    kq = 4 * (t & 7);
    cols = cols_;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + (t >> 3) + 32 * i;
      rowok[i] = m < Ks;
      base[i] = w + (int64_t)(rowok[i] ? m : 0) * ldw + kq;
    }
  }
  __device__ __forceinline__ void load(int ch) {
    const bool kok = ch * BK + kq < cols;
    const int kk = kok ? ch * BK : 0;  // keep the address inside the row; the value is masked below
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f32x4 v = *(const f32x4*)(base[i] + kk);
      const bool ok = kok && rowok[i];
      r[i] = v;
      okv[i] = ok;
    }
  }
  __device__ __forceinline__ void store(float* s) const {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float* d = s + kq * LD + (t >> 3) + 32 * i;
      const f32x4 v = masked(r[i], okv[i]);
      d[0] = v.x;
      d[LD] = v.y;
      d[2 * LD] = v.z;
      d[3 * LD] = v.w;
    }
  }
};

// B[kk][col] = x_t[tap kk of the column block's pixel][n], zero where the tap falls
// into the padding.  Each thread walks its four reduction rows kk = (c,r,s) with
// carry arithmetic (+32 per chunk), so no division or table sits in the loop.
struct FwdLoadB {
  static constexpr int LD = LDV;
  const float* xt;
  int base, h0, w0, H, W, C, R, S, HW, Np;
  int dc, dr, ds;         // (c,r,s) increments of one chunk
  int cc[4], rr[4], ss[4];
  bool cbok;
  f32x4 r[4];
  bool okv[4];  // value mask, applied when the registers go to LDS
  __device__ FwdLoadB(const Geo& g, const float* xt_, int ct) : xt(xt_) {
    const int t = threadIdx.x;
    const int vcq = t & 31;
    const int gcb = ct * 4 + (vcq >> 3);
    cbok = gcb < g.PQ * g.NB;
    const int pix = cbok ? gcb / g.NB : 0;
    const int nb = cbok ? gcb - pix * g.NB : 0;
    const int p = pix / g.Q, q = pix - p * g.Q;
    h0 = p * g.sh - g.ph;
    w0 = q * g.sw - g.pw;
    H = g.H; W = g.W; C = g.C; R = g.R; S = g.S; HW = g.HW; Np = g.Np;
    base = nb * 32 + 4 * (vcq & 7);
    dc = BK / g.RS;
    const int rem = BK - dc * g.RS;
    dr = rem / g.S;
    ds = rem - dr * g.S;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int kk = (t >> 5) + 8 * i;
      cc[i] = kk / g.RS;
      const int rs = kk - cc[i] * g.RS;
      rr[i] = rs / g.S;
      ss[i] = rs - rr[i] * g.S;
    }
  }
  __device__ __forceinline__ void load(int) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int hh = h0 + rr[i], vv = w0 + ss[i];
      const bool ok = cbok && cc[i] < C && (unsigned)hh < (unsigned)H && (unsigned)vv < (unsigned)W;
      const int off = ok ? (cc[i] * HW + hh * W + vv) * Np + base : 0;
      const f32x4 v = *(const f32x4*)(xt + off);
      r[i] = v;
      okv[i] = ok;
      // advance (c,r,s) by one chunk
      ss[i] += ds;
      if (ss[i] >= S) { ss[i] -= S; rr[i] += 1; }
      rr[i] += dr;
      if (rr[i] >= R) { rr[i] -= R; cc[i] += 1; }
      cc[i] += dc;
    }
  }
  __device__ __forceinline__ void store(float* s) const {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) *(f32x4*)(s + ((t >> 5) + 8 * i) * LD + 4 * (t & 31)) = masked(r[i], okv[i]);
  }
};

// y_t[k][pix][n] for the slice; one workgroup per 128 kernels x 4 column blocks.
__global__ __launch_bounds__(NT) void fwd_gemm_kernel(Geo g, const float* __restrict__ w, int ldw,
                                                      int wcols, const float* __restrict__ xt,
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
  FwdLoadA la(w, ldw, wcols, m0, g.Ks);
  FwdLoadB lb(g, xt, ct);
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
// A^T[k][c] = w_t[tap][k][c] (filters re-laid with c innermost, pitch Cp).
struct BwdDataLoadA {
  static constexpr int LD = LDV;
  const float* wt;
  const int* taps;
  int Ks, Cp, S, nkc, c, ti, kc;
  int64_t tapbase;
  f32x4 r[4];
  bool okv[4];  // value mask, applied when the registers go to LDS
  __device__ BwdDataLoadA(const Geo& g, const float* wt_, int Cp_, int m0, const int* taps_, int nkc_)
      : wt(wt_), taps(taps_), Ks(g.Ks), Cp(Cp_), S(g.S), nkc(nkc_), ti(0), kc(0), tapbase(0) {
    c = m0 + 4 * (threadIdx.x & 31);
  }
  __device__ __forceinline__ void set_tap() {
    const int e = taps[ti];
    const int tap = (e >> 16) * S + (e & 0xffff);
    tapbase = (int64_t)tap * Ks * Cp;
  }
  __device__ __forceinline__ void load(int) {
    if (kc == 0) set_tap();
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = kc * BK + (t >> 5) + 8 * i;
      const bool ok = k < Ks && c < Cp;
      const f32x4 v = *(const f32x4*)(wt + (ok ? tapbase + (int64_t)k * Cp + c : 0));
      r[i] = v;
      okv[i] = ok;
    }
    if (++kc == nkc) {
      kc = 0;
      ++ti;
    }
  }
  __device__ __forceinline__ void store(float* s) const {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) *(f32x4*)(s + ((t >> 5) + 8 * i) * LD + 4 * (t & 31)) = masked(r[i], okv[i]);
  }
};

// B[k][col] = dy_t[k][p][q][n] with (p,q) the output pixel whose window puts the
// current tap on the column block's input pixel; zero if there is none.
struct BwdDataLoadB {
  static constexpr int LD = LDV;
  const float* dyt;
  const int* taps;
  int Ks, nkc, ti, kc;
  int hp, vp, sh, sw, P, Q, PQNp, nboff, Np_;  // hp = h + pad_h, vp = v + pad_w of this thread's pixel
  int off;
  bool cbok, tapok;
  f32x4 r[4];
  bool okv[4];  // value mask, applied when the registers go to LDS
  __device__ BwdDataLoadB(const Geo& g, const float* dyt_, const int* perm, int ct, const int* taps_, int nkc_)
      : dyt(dyt_), taps(taps_), Ks(g.Ks), nkc(nkc_), ti(0), kc(0), off(0), tapok(false) {
    const int vcq = threadIdx.x & 31;
    const int gcb = ct * 4 + (vcq >> 3);
    cbok = gcb < g.HW * g.NB;
    const int sp = cbok ? gcb / g.NB : 0;
    const int nb = cbok ? gcb - sp * g.NB : 0;
    const int px = perm[sp];
    hp = px / g.W + g.ph;
    vp = px % g.W + g.pw;
    sh = g.sh;
    sw = g.sw;
    P = g.P;
    Q = g.Q;
    PQNp = g.PQ * g.Np;
    nboff = nb * 32 + 4 * (vcq & 7);
    Np_ = g.Np;
  }
  __device__ __forceinline__ void set_tap() {
    const int e = taps[ti];
    const int hr = hp - (e >> 16), vs = vp - (e & 0xffff);
    const int p = hr / sh, q = vs / sw;
    tapok = cbok && hr >= 0 && vs >= 0 && p * sh == hr && q * sw == vs && p < P && q < Q;
    off = (p * Q + q) * Np_ + nboff;
  }
  __device__ __forceinline__ void load(int) {
    if (kc == 0) set_tap();
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = kc * BK + (t >> 5) + 8 * i;
      const bool ok = tapok && k < Ks;
      const f32x4 v = *(const f32x4*)(dyt + (ok ? (int64_t)k * PQNp + off : 0));
      r[i] = v;
      okv[i] = ok;
    }
    if (++kc == nkc) {
      kc = 0;
      ++ti;
    }
  }
  __device__ __forceinline__ void store(float* s) const {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) *(f32x4*)(s + ((t >> 5) + 8 * i) * LD + 4 * (t & 31)) = masked(r[i], okv[i]);
  }
};

// dx_t[c][pixel][n]; column tiles follow the pixel order in perm (heaviest first).
__global__ __launch_bounds__(NT) void bwd_data_gemm_kernel(Geo g, const float* __restrict__ wt, int Cp,
                                                           const float* __restrict__ dyt,
                                                           const int* __restrict__ perm,
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
  BwdDataLoadA la(g, wt, Cp, m0, s_taps, nkc);
  BwdDataLoadB lb(g, dyt, perm, ct, s_taps, nkc);
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
// A[m][kk] = dy_t[m0+m][pix][n]: dense rows.
struct BwdWeightLoadA {
  static constexpr int LD = LDT;
  const float* base[4];
  bool rowok[4];
  f32x4 r[4];
  bool okv[4];  // value mask, applied when the registers go to LDS
  __device__ BwdWeightLoadA(const Geo& g, const float* dyt, int m0) {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = m0 + (t >> 3) + 32 * i;
      rowok[i] = m < g.Ks;
      base[i] = dyt + (int64_t)(rowok[i] ? m : 0) * g.PQ * g.Np + 4 * (t & 7);
    }
  }
  __device__ __forceinline__ void load(int ch) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f32x4 v = *(const f32x4*)(base[i] + (int64_t)ch * BK);
      r[i] = v;
      okv[i] = rowok[i];
    }
  }
  __device__ __forceinline__ void store(float* s) const {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float* d = s + 4 * (t & 7) * LD + (t >> 3) + 32 * i;
      const f32x4 v = masked(r[i], okv[i]);
      d[0] = v.x;
      d[LD] = v.y;
      d[2 * LD] = v.z;
      d[3 * LD] = v.w;
    }
  }
};

// B^T[j][kk] = x_t[c_j][p*sh-ph+r_j][q*sw-pw+s_j][n]; zero where tap j is in the padding.
struct BwdWeightLoadB {
  static constexpr int LD = LDT;
  const float* xt;
  int colbase[4], rj[4], sj[4];
  bool colok[4];
  int NB, Q, sh, sw, ph, pw, H, W, Np, nq;
  f32x4 r[4];
  bool okv[4];  // value mask, applied when the registers go to LDS
  __device__ BwdWeightLoadB(const Geo& g, const float* xt_, int j0) : xt(xt_) {
    const int t = threadIdx.x;
    NB = g.NB; Q = g.Q; sh = g.sh; sw = g.sw; ph = g.ph; pw = g.pw; H = g.H; W = g.W; Np = g.Np;
    nq = 4 * (t & 7);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = j0 + (t >> 3) + 32 * i;
      colok[i] = j < g.CRS;
      const int jj = colok[i] ? j : 0;
      const int c = jj / g.RS, rs = jj - c * g.RS;
      rj[i] = rs / g.S;
      sj[i] = rs - rj[i] * g.S;
      colbase[i] = c * g.HW * g.Np;
    }
  }
  __device__ __forceinline__ void load(int ch) {
    const int pix = ch / NB, nb = ch - pix * NB;
    const int p = pix / Q, q = pix - p * Q;
    const int h0 = p * sh - ph, v0 = q * sw - pw;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int hh = h0 + rj[i], vv = v0 + sj[i];
      const bool ok = colok[i] && (unsigned)hh < (unsigned)H && (unsigned)vv < (unsigned)W;
      const f32x4 v = *(const f32x4*)(xt + (ok ? colbase[i] + (hh * W + vv) * Np + nb * 32 + nq : 0));
      r[i] = v;
      okv[i] = ok;
    }
  }
  __device__ __forceinline__ void store(float* s) const {
    const int t = threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float* d = s + nq * LD + (t >> 3) + 32 * i;
      const f32x4 v = masked(r[i], okv[i]);
      d[0] = v.x;
      d[LD] = v.y;
      d[2 * LD] = v.z;
      d[3 * LD] = v.w;
    }
  }
};

// out[z][m][j] partial (or final when one split) weight gradients of the slice.
__global__ __launch_bounds__(NT) void bwd_weight_gemm_kernel(Geo g, const float* __restrict__ dyt,
                                                             const float* __restrict__ xt,
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
  BwdWeightLoadB lb(g, xt, j0);
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
