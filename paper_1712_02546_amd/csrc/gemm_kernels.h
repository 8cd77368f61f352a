// The three matrix-core passes.  Each is an implicit GEMM on 128x128 tiles (MI = 2; a last
// row tile of at most 64 rows is computed on 64x128 tiles, MI = 1, one of 65 to 96 rows on
// 96x128 tiles, MI = 3, by a launch of its own; see Shape<MI> in conv_common.h) whose 32-lane
// column blocks are "32 images at one pixel" (fwd, bwd_data) or 32 filter taps (bwd_weight);
// the operand loaders below are the only pass-specific code.
// A loader computes, per lane, the global address of the 16 bytes that lane moves
// into LDS for each of its wavefront's DMA loads per chunk (four for a 128-row or
// 128-column operand, three for 96 rows, two for 64; see the staging notes in
// conv_common.h for the row and col tile images).
#pragma once
#include "conv_common.h"

namespace cs {

// ---------------------------------------------------------------- forward ----
// A[m][kk] = w[k0+m0+m][kk]: rows of the filter matrix, col image.  The row pitch ldw is a
// multiple of BK and rows are zero past C*R*S, so no lane ever needs a mask: a lane's byte
// offset from the tile's first row is fixed and only the uniform base moves along the rows.
template <int MI_>
struct FwdLoadA {
  static constexpr bool COL = true;
  static constexpr int MI = MI_;   // tile shape (Shape<MI>)
  const char* tile;   // uniform: row m0 of the filter matrix
  const char* ub;     // uniform: tile + the chunk being issued
  unsigned off[Shape<MI>::NLOAD];
  __device__ FwdLoadA(const float* w, int ldw, int m0, int Ks) : tile((const char*)(w + (int64_t)m0 * ldw)) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < Shape<MI>::NLOAD; ++i) {
      const int kq4 = 4 * ((l & 7) ^ col_key(Shape<MI>::WROWS * wv + 8 * i + (l >> 3)));
      const int m = min(Shape<MI>::WROWS * wv + 8 * i + (l >> 3), Ks - 1 - m0);  // rows past the slice repeat the last one
      off[i] = ((unsigned)m * (unsigned)ldw + kq4) * 4u;
    }
  }
  // Chunks past the last one (live = false) re-read the row start, which is always there.
  __device__ __forceinline__ void begin(int ch, bool live) { ub = tile + (live ? ch : 0) * (BK * 4); }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {}
};

// B[kk][col] = x_t[tap kk of the column block's pixel][n] (row image), zero where the
// tap falls into the padding.  A zero page sits ZERO_PAGE_FLOATS in front of x_t and is the
// uniform base of every load; off_tab[kk] = byte offset of tap (c,r,s) from that base,
// rs_tab[kk] = (r<<16)|s (read only when the layer has padding).  Both are read with scalar
// loads one chunk ahead; a DMA load covers two consecutive reduction rows, one per half-wave,
// so a lane's offset is "its row's table entry + its pixel": three vector instructions.
template <bool PAD>
struct FwdLoadB {
  static constexpr bool COL = false;
  const char* zp;        // uniform: the zero page in front of x_t
  const CS_CONST int* off_tab;   // constant address space: read with scalar loads
  const CS_CONST int* rs_tab;
  i32x4 cur[2], nxt[2];   // offsets of rows 8*wv .. 8*wv+7 of the chunk being issued / the next one; uniform
  i32x4 cur_rs[2], nxt_rs[2];
  unsigned pixbase;      // byte offset of the lane's pixel, image block and 16-byte piece (may wrap below zero)
  int h0, w0, H, W;
  unsigned upmask;
  bool upper;
  __device__ FwdLoadB(const Geo& g, const float* xt, const int* tab, int entries, int ct, int ch0)
      : zp(opaque_uniform(xt - ZERO_PAGE_FLOATS)), off_tab((const CS_CONST int*)tab),
        rs_tab((const CS_CONST int*)tab + entries) {
    const int l = threadIdx.x & 63;
    const int cq = l & 31;
    // column blocks past the end are computed like block 0 and never stored
    const int gcb = ct * 4 + (cq >> 3) < g.PQ * g.NB ? ct * 4 + (cq >> 3) : 0;
    const int pix = gcb / g.NB;
    const int nb = gcb - pix * g.NB;
    const int p = pix / g.Q, q = pix - p * g.Q;
    h0 = p * g.sh - g.ph;
    w0 = q * g.sw - g.pw;
    H = g.H;
    W = g.W;
    pixbase = (unsigned)((h0 * g.W + w0) * g.Np + nb * 32 + 4 * (cq & 7)) * 4u;
    upper = l >= 32;
    upmask = upper ? ~0u : 0u;
    asm volatile("" : "+v"(upmask));
    fetch(ch0);
  }
  // Table rows past C*R*S repeat row 0 (the filter operand is zero there), and the table
  // runs three chunks past the end, so neither the tail nor the dummy chunks need a test.
  __device__ __forceinline__ void begin(int ch, bool) {
    cur[0] = nxt[0];
    cur[1] = nxt[1];
    if (PAD) {
      cur_rs[0] = nxt_rs[0];
      cur_rs[1] = nxt_rs[1];
    }
    fetch(ch + 1);
  }
  __device__ __forceinline__ void fetch(int ch) {   // rows 8*wv .. 8*wv+7 of chunk ch
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const CS_CONST i32x4* po = (const CS_CONST i32x4*)(off_tab + ch * BK + 8 * wv);
    nxt[0] = po[0];
    nxt[1] = po[1];
    if (PAD) {
      const CS_CONST i32x4* pr = (const CS_CONST i32x4*)(rs_tab + ch * BK + 8 * wv);
      nxt_rs[0] = pr[0];
      nxt_rs[1] = pr[1];
    }
  }
  static __device__ __forceinline__ int pick(const i32x4 (&v)[2], int r) { return v[r >> 2][r & 3]; }  // r: compile-time row 0..7
  __device__ __forceinline__ void issue(int i, float* dst) {
    // lower half-wave: row 2i, upper half-wave: row 2i+1.  Written as "a + ((b - a) & mask)"
    // with an opaque all-ones/all-zeros lane mask: two vector instructions, the difference is scalar.
    const unsigned a = (unsigned)pick(cur, 2 * i), b = (unsigned)pick(cur, 2 * i + 1);
    unsigned off = ((b - a) & upmask) + a + pixbase;
    if (PAD) {
      const unsigned ra = (unsigned)pick(cur_rs, 2 * i), rb = (unsigned)pick(cur_rs, 2 * i + 1);
      const int rs = (int)(ra + ((rb - ra) & upmask));   // same half-wave choice, again without a select
      const bool ok = ((unsigned)(h0 + (rs >> 16)) < (unsigned)H) & ((unsigned)(w0 + (rs & 0xffff)) < (unsigned)W);
      off = ok ? off : 0u;
    }
    dma16_uv(zp, off, dst);
  }
  __device__ __forceinline__ void end() {}
};

// Accumulator images in wavefront layout: element e = (i*NJ+j)*16+v of thread t at [e*NT + t].
template <int MI>
__device__ __forceinline__ void store_partial(float* slot, const f32x16 (&acc)[MI][Shape<MI>::NJ]) {
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < Shape<MI>::NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) slot[((i * Shape<MI>::NJ + j) * 16 + v) * NT + threadIdx.x] = acc[i][j][v];
}

// Sum of the scratch slots of tail tile tl, in run order, for the accumulator block stored as number blk.
__device__ __forceinline__ void gather_partials(const float* partial, const TailPlan& tp, int nch, int tl,
                                                int blk, f32x16& acc) {
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const int wfirst = (tl * nch) / tp.units;
  const int wlast = min(tp.nTailWg - 1, (tl * nch + nch - 1) / tp.units);
  for (int w = wfirst; w <= wlast; ++w) {
    const int slot = (w * tp.units) / nch == tl ? 0 : 1;   // a run's first tile uses slot 0, its second slot 1
    const float* p = partial + (int64_t)(w * 2 + slot) * TAIL_SLOT_FLOATS + blk * 16 * NT + threadIdx.x;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] += p[v * NT];
  }
}

// One workgroup's share of an equal-cost pass: a whole tile, or a run of the tail.
// body(L, ch_begin, ch_end, direct, slot) computes chunks [ch_begin, ch_end) of the tile at
// line position L and stores them as the final result (direct) or into a scratch slot.
template <class Body>
__device__ __forceinline__ void for_each_segment(const TailPlan& tp, int nch, Body&& body) {
  const int gid = blockIdx.x;
  const int gfull = grid_contiguous(tp.nFull);
  if (gid < gfull) {
    int L;
    if (line_contiguous(gid, tp.nFull, L)) body(L, 0, nch, true, 0);
    return;
  }
  int w;   // the runs of the tail are dealt to the XCDs in contiguous blocks too: neighbours share operand panels
  if (!line_contiguous(gid - gfull, tp.nTailWg, w)) return;
  int u0 = w * tp.units;
  const int u1 = min(u0 + tp.units, tp.nTail * nch);
  int tl = u0 / nch;
  int c = u0 - tl * nch;
  for (int slot = 0; slot < 2 && u0 < u1; ++slot) {
    const int ce = min(nch, c + (u1 - u0));
    body(tp.nFull + tl, c, ce, false, w * 2 + slot);
    u0 += ce - c;
    ++tl;
    c = 0;
  }
}

// Stores accumulator block (i,j) of this wavefront: 32 kernels x 32 images of one pixel.
// m0 = first row of the tile, MI = tile rows / 64.
template <int MI>
__device__ __forceinline__ void fwd_store_block(const Geo& g, float* __restrict__ yt, int m0, int ct, int i, int j,
                                                const f32x16& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int gcb = ct * 4 + Shape<MI>::colblk0(wave) + j;
  if (gcb >= g.PQ * g.NB) return;
  const int pix = gcb / g.NB, nb = gcb - pix * g.NB;
  const int n = nb * 32 + (lane & 31);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + Shape<MI>::row0(wave) + i * 32 + acc_row(v, lane);
    if (m < g.Ks) yt[((int64_t)m * g.PQ + pix) * g.Np + n] = acc[v];
  }
}

template <int MI>
__device__ __forceinline__ void fwd_store_tile(const Geo& g, float* __restrict__ yt, int m0, int ct,
                                               const f32x16 (&acc)[MI][Shape<MI>::NJ]) {
#pragma unroll
  for (int j = 0; j < Shape<MI>::NJ; ++j)
#pragma unroll
    for (int i = 0; i < MI; ++i) fwd_store_block<MI>(g, yt, m0, ct, i, j, acc[i][j]);
}

// y_t[k][pix][n] for rows mOrigin .. of the slice; a tile is 64*MI kernels x 4 column blocks
// and MB counts the row tiles of this launch.
template <bool PAD, int MI>
__global__ __launch_bounds__(NT) void fwd_gemm_kernel(Geo g, const float* __restrict__ w, int ldw,
                                                      const float* __restrict__ xt,
                                                      const int* __restrict__ tab, int entries,
                                                      float* __restrict__ yt, int mOrigin, int MB, int CT, int nch,
                                                      TailPlan tp, float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  for_each_segment(tp, nch, [&](int L, int cb, int ce, bool direct, int slot) {
    int mb, ct;
    tile_from_line(L, MB, CT, mb, ct);
    const int m0 = mOrigin + mb * Shape<MI>::ROWS;
    f32x16 acc[MI][Shape<MI>::NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < Shape<MI>::NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    FwdLoadA<MI> la(w, ldw, m0, g.Ks);
    FwdLoadB<PAD> lb(g, xt, tab, entries, ct, cb);
    gemm_mainloop(la, lb, cb, ce, smem, acc);
    if (direct) fwd_store_tile<MI>(g, yt, m0, ct, acc);
    else store_partial<MI>(partial + (int64_t)slot * TAIL_SLOT_FLOATS, acc);
  });
}

// Adds up the scratch slots of each tail tile and stores the tile.  grid = (nTail, MI*NJ): one
// workgroup per tile and accumulator block.
template <int MI>
__global__ __launch_bounds__(NT) void fwd_tail_fixup_kernel(Geo g, const float* __restrict__ partial,
                                                            float* __restrict__ yt, int mOrigin, int MB, int CT,
                                                            int nch, TailPlan tp) {
  const int bi = blockIdx.y / Shape<MI>::NJ, bj = blockIdx.y % Shape<MI>::NJ;
  f32x16 acc;
  gather_partials(partial, tp, nch, blockIdx.x, blockIdx.y, acc);
  int mb, ct;
  tile_from_line(tp.nFull + blockIdx.x, MB, CT, mb, ct);
  fwd_store_block<MI>(g, yt, mOrigin + mb * Shape<MI>::ROWS, ct, bi, bj, acc);
}

// --------------------------------------------------------- input gradient ----
// Reduction runs over (tap, k): only taps that reach the tile's pixels, k inner.
// Per tile, LDS holds the tap list s_taps[ti] = (r<<16)|s and, per tap and column
// block, s_tapoff[ti][cb] = offset of the matching output pixel inside dy_t, or -1.
// The (tap, k-chunk) counters are uniform and advance once per issue.
struct TapWalk {
  int ti, kc, nkc;
  __device__ TapWalk(int nkc_, int ch0) : ti(ch0 / nkc_), kc(ch0 - (ch0 / nkc_) * nkc_), nkc(nkc_) {}
  __device__ __forceinline__ void next() {   // branch-free carry
    ++kc;
    const int c = kc == nkc;
    kc = c ? 0 : kc;
    ti += c;
  }
};

// A[c][k] = w_t[tap][c][k] (filters re-laid tap-major with k innermost, pitch Ksp = 32*nkc,
// zero past Ks), col image, like the forward pass's filter operand: the uniform base is the
// chunk's (tap, k) position in the tile's first channel row, a lane's offset never changes.
template <int MI_>
struct BwdDataLoadA {
  static constexpr bool COL = true;
  static constexpr int MI = MI_;   // tile shape (Shape<MI>)
  const char* wt;     // uniform: w_t at channel m0 of tap 0
  const char* ub;     // uniform base of the chunk being issued
  const int* taps;
  unsigned off[Shape<MI>::NLOAD];
  unsigned tapBytes;  // one tap: C rows (a whole work copy is below 4 GiB)
  int tap;            // flat tap r*S+s of walk.ti, fetched one call ahead (uniform, held in a vector register)
  TapWalk walk;
  __device__ BwdDataLoadA(const Geo& g, const float* wt_, int Ksp, int m0, const int* taps_, int nkc_, int ch0)
      : wt((const char*)(wt_ + (int64_t)m0 * Ksp)), taps(taps_), tapBytes((unsigned)g.C * (unsigned)Ksp * 4u), walk(nkc_, ch0) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < Shape<MI>::NLOAD; ++i) {
      const int kq4 = 4 * ((l & 7) ^ col_key(Shape<MI>::WROWS * wv + 8 * i + (l >> 3)));
      const int c = min(Shape<MI>::WROWS * wv + 8 * i + (l >> 3), g.C - 1 - m0);   // channels past the end repeat the last one (never stored)
      off[i] = ((unsigned)c * (unsigned)Ksp + kq4) * 4u;
    }
    tap = taps[walk.ti];
  }
  __device__ __forceinline__ void begin(int, bool) {
    ub = wt + ((unsigned)__builtin_amdgcn_readfirstlane(tap) * tapBytes + (unsigned)walk.kc * (BK * 4u));
  }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {
    walk.next();
    tap = taps[walk.ti];   // entries past the list are allocated and hold tap 0, so this stays in bounds
  }
};

// B[k][col] = dy_t[k][pixel][n] (row image; Ksp rows of P*Q+1 pixels, the extra pixel and
// the rows past Ks are zero) with `pixel` the output pixel whose window puts the current tap
// on the column block's input pixel, or the zero pixel if there is none.  The uniform base
// is the k row of each load; a lane adds its half-wave's row, its block's pixel and its piece.
struct BwdDataLoadB {
  static constexpr bool COL = false;
  const char* dyt;    // uniform
  const char* ub;     // uniform: rows of the chunk being issued
  const int* tapoff;
  unsigned pairBytes; // two k rows
  unsigned kBytes;    // one k row (a whole work copy is below 4 GiB)
  unsigned lane_const, off;
  int cb, wv8, toff;   // toff = tapoff[walk.ti][cb], fetched one call ahead
  TapWalk walk;
  __device__ BwdDataLoadB(const Geo& g, const float* dyt_, const int* tapoff_, int nkc_, int ch0)
      : dyt((const char*)dyt_), tapoff(tapoff_), walk(nkc_, ch0) {
    const int l = threadIdx.x & 63;
    const int cq = l & 31;
    const int pitchK = (g.PQ + 1) * g.Np;
    kBytes = (unsigned)pitchK * 4u;
    pairBytes = 2u * kBytes;
    cb = cq >> 3;
    wv8 = 8 * __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    lane_const = (unsigned)((l >> 5) * pitchK + 4 * (cq & 7)) * 4u;
    toff = tapoff[walk.ti * 4 + cb];
  }
  __device__ __forceinline__ void begin(int, bool) {
    ub = dyt + (unsigned)(walk.kc * BK + wv8) * kBytes;
    off = lane_const + (unsigned)toff * 4u;
  }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub + (unsigned)i * pairBytes, off, dst); }
  __device__ __forceinline__ void end() {
    walk.next();
    toff = tapoff[walk.ti * 4 + cb];
  }
};

// Even sharing of the input-gradient pass (tiles of unequal cost).  The column tiles, pixels
// by decreasing tap count, form a line on which tile ct covers chunks pre[ct] .. pre[ct+1]
// (its taps times the k-chunks; the ordering kernel writes pre and the line's length pre[CT]).
// The line is cut into nRuns equal runs (run_units), and each run is computed by MB
// workgroups, one per row tile (nWg = nRuns * MB): workgroup run*MB+mb computes row tile mb of
// the column tiles inside its run whole and of the (at most two) tiles that stick out at either
// end partially, into scratch slot 2*wg (the tile its run starts in) or 2*wg+1; a fix-up kernel
// adds the slots of a cut tile in run order.  enabled = 0: one workgroup per tile, heaviest
// first (tile_dealt).
struct RunPlan {
  int enabled, nRuns, nWg;
};

// Length of the equal runs a line of `total` chunks is cut into for nRuns groups: whole taps
// (nkc chunks) when that leaves less than 3 % of the slots idle, any number of chunks
// otherwise (few, long taps); at least 8.
__device__ __forceinline__ int run_units(int total, int nkc, int nRuns) {
  int units = ((total / nkc + nRuns - 1) / nRuns) * nkc;
  if ((float)total < 0.97f * (float)nRuns * (float)units) units = (total + nRuns - 1) / nRuns;
  return max(units, 8);
}

// m0 = first channel of the tile, MI = tile rows / 64.
template <int MI>
__device__ __forceinline__ void bwd_data_store_block(const Geo& g, float* __restrict__ dxt,
                                                     const int* __restrict__ perm, int m0, int ct, int i, int j,
                                                     const f32x16& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int gcb = ct * 4 + Shape<MI>::colblk0(wave) + j;
  if (gcb >= g.HW * g.NB) return;
  const int sp = gcb / g.NB, nb = gcb - sp * g.NB;
  const int px = perm[sp];
  const int n = nb * 32 + (lane & 31);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int c = m0 + Shape<MI>::row0(wave) + i * 32 + acc_row(v, lane);
    if (c < g.C) dxt[((int64_t)c * g.HW + px) * g.Np + n] = acc[v];
  }
}

// dx_t[c][pixel][n] for channels mOrigin .. in MB row tiles of 64*MI channels; column tiles
// follow the pixel order in perm.
template <int MI>
__global__ __launch_bounds__(NT) void bwd_data_gemm_kernel(Geo g, const float* __restrict__ wt, int Ksp,
                                                           const float* __restrict__ dyt,
                                                           const int* __restrict__ perm,
                                                           const int* __restrict__ pre,
                                                           float* __restrict__ dxt, int mOrigin, int MB, int CT,
                                                           RunPlan rp, float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  int* s_taps = (int*)(smem + 4 * TILE_F);     // [RS + 3]: the loaders run up to three entries past the list
  int* s_tapoff = s_taps + g.RS + 3;           // [RS + 3][4]
  __shared__ int s_ntaps;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nkc = (g.Ks + BK - 1) / BK;

  // Chunks [c0, c1) of tile (mb, ct), stored as the result (direct) or into a scratch slot.
  auto segment = [&](int mb, int ct, int c0, int c1, bool direct, int slot) {
    // Taps that reach at least one of the tile's (up to four) pixels, in (r,s) order, and
    // for each of them where it lands in dy_t for every column block.
    if (wave == 0) {
      int hp[4], vp[4], nbo[4];
      bool ok[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int gcb = ct * 4 + j;
        ok[j] = gcb < g.HW * g.NB;
        const int sp = ok[j] ? gcb / g.NB : 0;
        const int px = perm[sp];
        nbo[j] = ok[j] ? (gcb - sp * g.NB) * 32 : 0;
        hp[j] = px / g.W + g.ph;
        vp[j] = px % g.W + g.pw;
      }
      int cnt = 0;
      for (int b = 0; b < g.RS; b += 64) {
        const int tp = b + lane;
        const int rr = tp / g.S, ss = tp - rr * g.S;
        bool any = false;
        int offs[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int hr = hp[j] - rr, vs = vp[j] - ss;
          const int p = hr / g.sh, q = vs / g.sw;
          const bool hit = tp < g.RS && ok[j] && hr >= 0 && vs >= 0 && p * g.sh == hr && q * g.sw == vs &&
                           p < g.P && q < g.Q;
          offs[j] = (hit ? p * g.Q + q : g.PQ) * g.Np + nbo[j];   // no hit: the zero pixel
          any |= hit;
        }
        const unsigned long long mask = __ballot(any);
        if (any) {
          const int pos = cnt + __popcll(mask & ((1ull << lane) - 1ull));
          s_taps[pos] = tp;   // flat r*S+s
#pragma unroll
          for (int j = 0; j < 4; ++j) s_tapoff[pos * 4 + j] = offs[j];
        }
        cnt += __popcll(mask);
      }
      if (lane < 12) s_tapoff[cnt * 4 + lane] = g.PQ * g.Np;   // the entries the loaders fetch after the last tap
      if (lane < 3) s_taps[cnt + lane] = 0;
      if (lane == 0) s_ntaps = cnt;
    }
    __syncthreads();
    const int nchunks = s_ntaps * nkc;
    const int cb = min(c0, nchunks), ce = min(c1, nchunks);
    const int m0 = mOrigin + mb * Shape<MI>::ROWS;
    f32x16 acc[MI][Shape<MI>::NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < Shape<MI>::NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    BwdDataLoadA<MI> la(g, wt, Ksp, m0, s_taps, nkc, cb);
    BwdDataLoadB lb(g, dyt, s_tapoff, nkc, cb);
    gemm_mainloop(la, lb, cb, ce, smem, acc);
    if (direct) {
#pragma unroll
      for (int j = 0; j < Shape<MI>::NJ; ++j)
#pragma unroll
        for (int i = 0; i < MI; ++i) bwd_data_store_block<MI>(g, dxt, perm, m0, ct, i, j, acc[i][j]);
    } else {
      store_partial<MI>(partial + (int64_t)slot * TAIL_SLOT_FLOATS, acc);
    }
    __syncthreads();   // the next segment rewrites the tap list
  };

  if (!rp.enabled) {
    int mb, ct;
    if (!tile_dealt(blockIdx.x, MB, CT, mb, ct)) return;
    segment(mb, ct, 0, 0x7fffffff, true, 0);
    return;
  }

  // run mode: workgroups are dealt to the XCDs in contiguous blocks; workgroup w = run * MB + row tile
  const int wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  if (wg >= rp.nWg) return;
  const int run = wg / MB, mb = wg - run * MB;
  const int total = pre[CT], units = run_units(total, nkc, rp.nRuns);
  if ((int64_t)run * units >= total) return;
  int pos = run * units;
  const int end = min(pos + units, total);
  // the tile that holds pos: pre[ct] <= pos < pre[ct+1]
  int ct = 0;
  for (int hi = CT; hi - ct > 1;) {
    const int mid = (ct + hi) >> 1;
    if (pre[mid] <= pos) ct = mid; else hi = mid;
  }
  int c = pos - pre[ct];
  bool first = true;
  for (; pos < end && ct < CT; ++ct) {
    const int len = pre[ct + 1] - pre[ct];
    const int ce = min(len, c + (end - pos));
    segment(mb, ct, c, ce, c == 0 && ce == len, wg * 2 + (first ? 0 : 1));
    pos += ce - c;
    c = 0;
    first = false;
  }
}

// Adds up the scratch slots of every tile that was cut by a run boundary.  grid = (CT*MB, MI*NJ);
// nkc and nRuns as in the kernel that wrote the slots.
template <int MI>
__global__ __launch_bounds__(NT) void bwd_data_fixup_kernel(Geo g, const int* __restrict__ perm,
                                                            const int* __restrict__ pre,
                                                            const float* __restrict__ partial,
                                                            float* __restrict__ dxt, int mOrigin, int MB, int CT,
                                                            int nkc, int nRuns) {
  const int ct = blockIdx.x / MB, mb = blockIdx.x - ct * MB;
  const int units = run_units(pre[CT], nkc, nRuns);
  const int a = pre[ct], b = pre[ct + 1];   // the tile's stretch of the line
  const int r0 = a / units, r1 = (b - 1) / units;
  if (r0 == r1) return;   // inside one run: stored directly
  const int bi = blockIdx.y / Shape<MI>::NJ, bj = blockIdx.y % Shape<MI>::NJ;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  for (int r = r0; r <= r1; ++r) {
    const int slot = r * units >= a ? 0 : 1;   // a run that starts inside the tile used its first slot
    const float* p = partial + (int64_t)((r * MB + mb) * 2 + slot) * TAIL_SLOT_FLOATS + blockIdx.y * 16 * NT + threadIdx.x;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] += p[v * NT];
  }
  bwd_data_store_block<MI>(g, dxt, perm, mOrigin + mb * Shape<MI>::ROWS, ct, bi, bj, acc);
}

// ---------------------------------------------------------- weight gradient ----
// Reduction index = (output pixel, image block, image): chunk ch covers output pixel
// ch / NB, images nb*32 .. nb*32+31 with nb = ch % NB.
// A[m][kk] = dy_t[m0+m][ch*32 + kk]: rows of dy_t, col image.  A lane's offset from the
// tile's first row never changes; the uniform base advances by one chunk.
template <int MI_>
struct BwdWeightLoadA {
  static constexpr bool COL = true;
  static constexpr int MI = MI_;   // tile shape (Shape<MI>)
  const char* tile;   // uniform: row m0 of dy_t
  const char* ub;     // uniform: tile + the chunk being issued
  unsigned off[Shape<MI>::NLOAD];
  int first, stride;  // step i of the walk is chunk first + i*stride
  __device__ BwdWeightLoadA(const Geo& g, const float* dyt, int m0, int first_, int stride_)
      : tile((const char*)(dyt + (int64_t)m0 * g.PQ * g.Np)), first(first_), stride(stride_) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < Shape<MI>::NLOAD; ++i) {
      const int kq4 = 4 * ((l & 7) ^ col_key(Shape<MI>::WROWS * wv + 8 * i + (l >> 3)));
      const int m = min(Shape<MI>::WROWS * wv + 8 * i + (l >> 3), g.Ks - 1 - m0);  // rows past the slice repeat the last one
      off[i] = ((unsigned)m * (unsigned)(g.PQ * g.Np) + kq4) * 4u;
    }
  }
  __device__ __forceinline__ void begin(int i, bool live) { ub = tile + (int64_t)(live ? first + i * stride : 0) * (BK * 4); }  // dummy: chunk 0
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {}
};

// B^T[j][kk] = x_t[c_j][p*sh-ph+r_j][q*sw-pw+s_j][n] (col image); zero where tap j is in
// the padding.  Columns j past C*R*S are computed like column 0 and never stored.  The
// chunk's output pixel (p,q) and image block nb are uniform counters.  Without padding the
// window origin goes into the uniform base and a lane's offset is its constant column
// offset; with padding the base is the zero page in front of x_t, which out-of-range taps read.
template <bool PAD>
struct BwdWeightLoadB {
  static constexpr bool COL = true;
  const char* xt;        // uniform; a zero page sits ZERO_PAGE_FLOATS in front of x_t
  const char* ub;        // uniform base of the chunk being issued
  unsigned coff[4];      // bytes
  int rj[4], sj[4];
  int NB, Q, sh, sw, ph, pw, H, W, Np;
  int p, q, nb;          // uniform position of the next chunk to issue
  int dp, dq, dnb;       // one step of the walk (stride chunks) as a (p, q, nb) increment
  int h0, v0;            // uniform, of the chunk being issued
  unsigned uoff;
  __device__ BwdWeightLoadB(const Geo& g, const float* xt_, int j0, int ch0, int stride)
      : xt(PAD ? opaque_uniform(xt_ - ZERO_PAGE_FLOATS) : (const char*)xt_) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    NB = g.NB; Q = g.Q; sh = g.sh; sw = g.sw; ph = g.ph; pw = g.pw; H = g.H; W = g.W; Np = g.Np;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int kq4 = 4 * ((l & 7) ^ col_key(8 * i + (l >> 3)));
      const int j = j0 + 32 * wv + 8 * i + (l >> 3);
      const int jj = j < g.CRS ? j : 0;
      const int c = jj / g.RS, rs = jj - c * g.RS;
      rj[i] = rs / g.S;
      sj[i] = rs - rj[i] * g.S;
      coff[i] = (unsigned)(c * g.HW * g.Np + (rj[i] * g.W + sj[i]) * g.Np + kq4 + (PAD ? ZERO_PAGE_FLOATS : 0)) * 4u;
    }
    const int pix = ch0 / NB;
    nb = ch0 - pix * NB;
    p = pix / Q;
    q = pix - p * Q;
    const int dpix = stride / NB;
    dnb = stride - dpix * NB;
    dp = dpix / Q;
    dq = dpix - dp * Q;
  }
  __device__ __forceinline__ void begin(int, bool live) {
    h0 = live ? p * sh - ph : 0;       // the dummy issue re-reads the first pixel
    v0 = live ? q * sw - pw : 0;
    const int u = (h0 * W + v0) * Np + (live ? nb * 32 : 0);
    if (PAD) uoff = (unsigned)u * 4u;          // may wrap below zero; the sum with coff does not
    else ub = xt + (int64_t)u * 4;
  }
  __device__ __forceinline__ void issue(int i, float* dst) {
    if (PAD) {
      const bool ok = ((unsigned)(h0 + rj[i]) < (unsigned)H) & ((unsigned)(v0 + sj[i]) < (unsigned)W);
      unsigned o = ok ? coff[i] + uoff : 0u;
      dma16_uv(xt, o, dst);
    } else {
      dma16_uv(ub, coff[i], dst);
    }
  }
  __device__ __forceinline__ void end() {   // branch-free carry: (nb, q, p) += one step
    nb += dnb;
    const int cq = nb >= NB;
    nb -= cq ? NB : 0;
    q += dq + cq;
    const int cp = q >= Q;
    q -= cp ? Q : 0;
    p += dp + cp;
  }
};

// m0 = first row of the tile, MI = tile rows / 64; row m goes to row m - rowBase of `o`.
template <int MI>
__device__ __forceinline__ void bwd_weight_store_block(const Geo& g, float* __restrict__ o, int m0, int rowBase,
                                                       int ct, int i, int j, const f32x16& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = ct * BN + Shape<MI>::col0(wave) + j * 32 + (lane & 31);
  if (col >= g.CRS) return;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + Shape<MI>::row0(wave) + i * 32 + acc_row(v, lane);
    if (m < g.Ks) o[(int64_t)(m - rowBase) * g.CRS + col] = acc[v];
  }
}

template <int MI>
__device__ __forceinline__ void bwd_weight_store_tile(const Geo& g, float* __restrict__ o, int m0, int rowBase, int ct,
                                                      const f32x16 (&acc)[Shape<MI>::RB][Shape<MI>::NJ]) {
#pragma unroll
  for (int j = 0; j < Shape<MI>::NJ; ++j)
#pragma unroll
    for (int i = 0; i < Shape<MI>::RB; ++i) bwd_weight_store_block<MI>(g, o, m0, rowBase, ct, i, j, acc[i][j]);
}

// out[z][m][j]: partial (or final when one split) weight gradients of the slice.  Either
// splits = 1 and tp shares out the tail tiles, or (small outputs) the reduction is split:
// the tiles * splits work items (split-major) are dealt to the XCDs in contiguous blocks, so
// that every XCD has work whatever the tile count and the tiles of one split, which share
// operand rows, follow each other on one XCD.  grid = grid_contiguous(tiles * splits).  Split z
// takes chunks z, z + splits, z + 2*splits, ...: the workgroups of all splits run side by
// side, so together they read a contiguous stretch of every operand row at any moment.
template <bool PAD, int MI>
__global__ __launch_bounds__(NT) void bwd_weight_gemm_kernel(Geo g, const float* __restrict__ dyt,
                                                             const float* __restrict__ xt,
                                                             float* __restrict__ out, int64_t splitStride,
                                                             int mOrigin, int rowBase, int MB, int CT, int nch,
                                                             int splits, TailPlan tp, float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  int z = 0, Lsplit = 0;
  if (splits > 1) {
    const int tiles = MB * CT;
    int item;
    if (!line_contiguous(blockIdx.x, tiles * splits, item)) return;
    z = item / tiles;
    Lsplit = item - z * tiles;
  }
  float* o = out + (int64_t)z * splitStride;
  auto body = [&](int L, int cb, int ce, bool direct, int slot) {
    int mb, ct;
    tile_from_line(L, MB, CT, mb, ct);
    const int m0 = mOrigin + mb * Shape<MI>::ROWS;
    if (direct) {   // a whole tile: every chunk of this split
      cb = 0;
      ce = (nch - z + splits - 1) / splits;
    }
    f32x16 acc[MI][Shape<MI>::NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < Shape<MI>::NJ; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    BwdWeightLoadA<MI> la(g, dyt, m0, z, splits);
    BwdWeightLoadB<PAD> lb(g, xt, ct * BN, z + cb * splits, splits);
    gemm_mainloop(la, lb, cb, ce, smem, acc);
    if (direct) bwd_weight_store_tile<MI>(g, o, m0, rowBase, ct, acc);
    else store_partial<MI>(partial + (int64_t)slot * TAIL_SLOT_FLOATS, acc);
  };
  if (splits > 1) {
    body(Lsplit, 0, 0, true, 0);
    return;
  }
  for_each_segment(tp, nch, body);
}

// grid = (nTail, MI*NJ)
template <int MI>
__global__ __launch_bounds__(NT) void bwd_weight_tail_fixup_kernel(Geo g, const float* __restrict__ partial,
                                                                   float* __restrict__ out, int mOrigin, int rowBase,
                                                                   int MB, int CT, int nch, TailPlan tp) {
  const int bi = blockIdx.y / Shape<MI>::NJ, bj = blockIdx.y % Shape<MI>::NJ;
  f32x16 acc;
  gather_partials(partial, tp, nch, blockIdx.x, blockIdx.y, acc);
  int mb, ct;
  tile_from_line(tp.nFull + blockIdx.x, MB, CT, mb, ct);
  bwd_weight_store_block<MI>(g, out, mOrigin + mb * Shape<MI>::ROWS, rowBase, ct, bi, bj, acc);
}

}  // namespace cs
