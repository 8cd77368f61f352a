// Pixel order of the input-gradient pass, written as the phases of one workgroup.
//
// The H*W input pixels are sorted by decreasing tap count (a counting sort; no atomics in the
// placement, so the order is the same on every run): perm[position] = pixel.  The taps that
// reach a pixel are (row taps reaching h) x (column taps reaching v); along an axis they form
// an arithmetic progression with the stride as step, named by its length (a for rows, b for
// columns) and its first tap.  The tap count is a*b.  Pixels with the same count are ordered
// by a, then by the first row tap, then by the first column tap, so that pixels with the same
// set of taps are neighbours (column tiles that hold several pixels then walk no tap in
// vain), and inside such a group by the rank of the row and of the column in their classes:
// a pixel's position is a closed form of per-row and per-column ranks and class sizes, no
// loop over the image.  Pixels no tap reaches (a*b = 0) come last: whole rows with a = 0
// first, then the columns with b = 0 of the other rows.
//
// With `pre` given the CT column tiles (four blocks of 32 images each, blocks numbered
// position-major in the new order) are also laid on a line: a tile is as many chunks long as
// nkc times the number of taps that reach any of its pixels (at least one), pre[ct] is where
// tile ct starts and pre[CT] the length of the line.
//
// Every phase is a function of (thread, thread count) that touches the tables only through
// the Tables pointers; the kernel runs the phases with a workgroup barrier between them, and
// a host build can run them thread after thread with bounds-checked tables.  Table extents
// are functions of R, S, H, W alone (no table is indexed by a product of class keys):
//   bins   R*S + 2   pixels per tap count, then first position per tap count
//   rowCnt R + 1     rows per a           colCnt S + 1   columns per b
//   part   threads   per-thread sums of tile lengths
//   axes   6*H + 5*W per-row and per-column ranks (axes_ints)
#pragma once
#include "geo.h"

#if defined(__HIPCC__)
#define CS_PO_FN __host__ __device__ inline
#else
#define CS_PO_FN inline
#endif

namespace cs {
namespace po {

constexpr int MAX_RS = 1024;            // the library's limit on R*S (hence on R and on S)
constexpr int BINS = MAX_RS + 2;
constexpr int AXIS_CNT = MAX_RS + 2;
constexpr int THREADS = 1024;
constexpr int AXES_LDS = 6144;          // ints of per-axis tables kept in LDS; larger images use global scratch

CS_PO_FN int axes_ints(int H, int W) { return 6 * H + 5 * W; }

template <class P>
struct Tables {
  P bins, rowCnt, colCnt, part, axes;
  P perm;   // H*W
  P pre;    // CT + 1 (used only when lengths are wanted)
};

// `len` ints of a table from `off` on.  A host build with checked tables supplies its own overload.
CS_PO_FN int* view(int* base, int off, int) { return base + off; }

template <class P>
struct Axes {   // views into Tables::axes
  P nrow, rowKey, rowRank, nzRank, rowLess, rowSame, ncol, colKey, colRank, colLess, colSame;
  CS_PO_FN Axes(const P& b, int H, int W)
      : nrow(view(b, 0, H)), rowKey(view(b, H, H)), rowRank(view(b, 2 * H, H)), nzRank(view(b, 3 * H, H)),
        rowLess(view(b, 4 * H, H)), rowSame(view(b, 5 * H, H)), ncol(view(b, 6 * H, W)),
        colKey(view(b, 6 * H + W, W)), colRank(view(b, 6 * H + 2 * W, W)), colLess(view(b, 6 * H + 3 * W, W)),
        colSame(view(b, 6 * H + 4 * W, W)) {}
};

template <class Ref>
CS_PO_FN void add_to(Ref&& r, int v) {
#if defined(__HIP_DEVICE_COMPILE__)
  atomicAdd(&r, v);   // counts only: the sums do not depend on the order
#else
  r += v;
#endif
}

// Taps along one axis that reach coordinate x (input extent irrelevant: x is in range):
// count and first tap of {t in [0,F): (x + pad - t) >= 0, divisible by stride, quotient < O}.
CS_PO_FN void axis_taps(int x, int pad, int F, int stride, int O, int& n, int& first) {
  n = 0;
  first = 0;
  for (int t = F - 1; t >= 0; --t) {
    const int d = x + pad - t;
    if (d >= 0 && d % stride == 0 && d / stride < O) {
      ++n;
      first = t;
    }
  }
}

// Phase 1: clear the counters; tap progression (length, class key) of every row and column.
template <class P>
CS_PO_FN void phase_axes(const Geo& g, const Tables<P>& t, int tid, int T) {
  const Axes<P> ax(t.axes, g.H, g.W);
  for (int i = tid; i <= g.RS + 1; i += T) t.bins[i] = 0;
  for (int i = tid; i <= g.R; i += T) t.rowCnt[i] = 0;
  for (int i = tid; i <= g.S; i += T) t.colCnt[i] = 0;
  for (int h = tid; h < g.H; h += T) {
    int n, first;
    axis_taps(h, g.ph, g.R, g.sh, g.P, n, first);
    ax.nrow[h] = n;
    ax.rowKey[h] = n * g.R + first;
  }
  for (int v = tid; v < g.W; v += T) {
    int n, first;
    axis_taps(v, g.pw, g.S, g.sw, g.Q, n, first);
    ax.ncol[v] = n;
    ax.colKey[v] = n * g.S + first;
  }
}

// Phase 2: per row (column): rank inside its class, rows of the same length with a smaller
// key, size of its class; rows per length.
template <class P>
CS_PO_FN void phase_ranks(const Geo& g, const Tables<P>& t, int tid, int T) {
  const Axes<P> ax(t.axes, g.H, g.W);
  for (int h = tid; h < g.H; h += T) {
    const int key = ax.rowKey[h], a = ax.nrow[h];
    int rank = 0, nz = 0, less = 0, same = 0;
    for (int hh = 0; hh < g.H; ++hh) {
      const int k2 = ax.rowKey[hh];
      const bool eq = k2 == key;
      same += eq;
      rank += eq && hh < h;
      nz += hh < h && ax.nrow[hh] > 0;
      less += ax.nrow[hh] == a && k2 < key;
    }
    ax.rowRank[h] = rank;
    ax.nzRank[h] = nz;
    ax.rowLess[h] = less;
    ax.rowSame[h] = same;
    add_to(t.rowCnt[a], 1);
  }
  for (int v = T - 1 - tid; v < g.W; v += T) {   // from the last thread down: other wavefronts than the rows'
    const int key = ax.colKey[v], b = ax.ncol[v];
    int rank = 0, less = 0, same = 0;
    for (int vv = 0; vv < g.W; ++vv) {
      const int k2 = ax.colKey[vv];
      const bool eq = k2 == key;
      same += eq;
      rank += eq && vv < v;
      less += ax.ncol[vv] == b && k2 < key;
    }
    ax.colRank[v] = rank;
    ax.colLess[v] = less;
    ax.colSame[v] = same;
    add_to(t.colCnt[b], 1);
  }
}

// Phase 3: pixels per tap count.
template <class P>
CS_PO_FN void phase_bins(const Geo& g, const Tables<P>& t, int tid, int T) {
  for (int i = tid; i < (g.R + 1) * (g.S + 1); i += T) {
    const int a = i / (g.S + 1), b = i - a * (g.S + 1);
    add_to(t.bins[a * b], t.rowCnt[a] * t.colCnt[b]);
  }
}

// Phase 4 (one thread): first position of every tap count, heaviest first.
template <class P>
CS_PO_FN void phase_scan_bins(const Geo& g, const Tables<P>& t, int tid, int) {
  if (tid != 0) return;
  int run = 0;
  for (int wgt = g.RS; wgt >= 0; --wgt) {
    const int cnt = t.bins[wgt];
    t.bins[wgt] = run;
    run += cnt;
  }
}

// Phase 5: every pixel's position.
template <class P>
CS_PO_FN void phase_place(const Geo& g, const Tables<P>& t, int tid, int T) {
  const Axes<P> ax(t.axes, g.H, g.W);
  for (int px = tid; px < g.HW; px += T) {
    const int h = px / g.W, v = px - h * g.W;
    const int a = ax.nrow[h], b = ax.ncol[v];
    const int wgt = a * b;
    int pos;
    if (wgt > 0) {
      int before = 0;
      for (int a2 = 1; a2 < a; ++a2) {   // groups with the same count and a smaller a
        const int q = wgt / a2;
        if (q * a2 == wgt && q <= g.S) before += t.rowCnt[a2] * t.colCnt[q];
      }
      before += ax.rowLess[h] * t.colCnt[b];     // same a, earlier first row tap
      before += ax.rowSame[h] * ax.colLess[v];   // same rows, earlier first column tap
      pos = t.bins[wgt] + before + ax.rowRank[h] * ax.colSame[v] + ax.colRank[v];
    } else if (a == 0) {
      pos = t.bins[0] + ax.rowRank[h] * g.W + v;
    } else {
      pos = t.bins[0] + t.rowCnt[0] * g.W + ax.nzRank[h] * t.colCnt[0] + ax.colRank[v];
    }
    t.perm[pos] = px;
  }
}

// The contiguous stretch of tiles thread tid measures.
CS_PO_FN void tile_stretch(int CT, int tid, int T, int& t0, int& t1) {
  const int per = (CT + T - 1) / T;
  t0 = tid * per < CT ? tid * per : CT;
  t1 = t0 + per < CT ? t0 + per : CT;
}

// Common elements of two arithmetic progressions with the same step: {f1 + i*step, i < n1} and {f2 + i*step, i < n2}.
CS_PO_FN int common_taps(int f1, int n1, int f2, int n2, int step) {
  if (n1 <= 0 || n2 <= 0 || (f1 - f2) % step != 0) return 0;
  const int lo = f1 > f2 ? f1 : f2;
  const int l1 = f1 + (n1 - 1) * step, l2 = f2 + (n2 - 1) * step;
  const int hi = l1 < l2 ? l1 : l2;
  return hi >= lo ? (hi - lo) / step + 1 : 0;
}

// Phase 6: length of every tile into pre[ct+1], the thread's sum into part[tid].  A column tile
// is bpt (4 or 8) consecutive column blocks.
constexpr int MAX_BPT = 8;
template <class P>
CS_PO_FN void phase_lengths(const Geo& g, const Tables<P>& t, int CT, int nkc, int bpt, int tid, int T) {
  const Axes<P> ax(t.axes, g.H, g.W);
  int t0, t1;
  tile_stretch(CT, tid, T, t0, t1);
  int sum = 0;
  const bool one_pixel = g.NB % bpt == 0;   // every tile lies inside one pixel: its taps are a*b
  for (int ct = t0; ct < t1; ++ct) {
    int taps = 0;
    if (one_pixel) {
      const int px = t.perm[ct / (g.NB / bpt)];
      taps = ax.nrow[px / g.W] * ax.ncol[px % g.W];
    } else {
      // The tile's distinct pixels, each with its row and column taps as arithmetic progressions (first tap,
      // count; the step is the stride).  One or two pixels (the usual case) have a closed form; for more the taps
      // are walked once, every progression with a running "next tap": no division per tap and pixel.
      int fr[MAX_BPT], na[MAX_BPT], fs[MAX_BPT], nb[MAX_BPT], np = 0;
      for (int j = 0; j < bpt; ++j) {
        const int gcb = ct * bpt + j;
        if (gcb >= g.HW * g.NB) break;
        const int sp = gcb / g.NB;
        if (j > 0 && sp == (gcb - 1) / g.NB) continue;
        const int px = t.perm[sp];
        const int h = px / g.W, v = px - h * g.W;
        const int a = ax.nrow[h], b = ax.ncol[v];
        const int first_r = ax.rowKey[h] - a * g.R, first_s = ax.colKey[v] - b * g.S;
        for (int k = 0; k < MAX_BPT; ++k)
          if (k == np) { na[k] = a; fr[k] = first_r; nb[k] = b; fs[k] = first_s; }
        ++np;
      }
      if (np == 1) {
        taps = na[0] * nb[0];
      } else if (np == 2) {   // |R1 x S1| + |R2 x S2| - |R1 & R2| * |S1 & S2|
        taps = na[0] * nb[0] + na[1] * nb[1] -
               common_taps(fr[0], na[0], fr[1], na[1], g.sh) * common_taps(fs[0], nb[0], fs[1], nb[1], g.sw);
      } else {
        // (loops over all MAX_BPT entries with a test, so that a GPU build keeps the small arrays in registers)
        for (int j = np; j < MAX_BPT; ++j) { na[j] = 0; nb[j] = 0; fr[j] = 0; fs[j] = 0; }
        int nr[MAX_BPT], ir[MAX_BPT];
        for (int j = 0; j < MAX_BPT; ++j) { nr[j] = fr[j]; ir[j] = 0; }
        for (int r = 0; r < g.R; ++r) {
          unsigned rowhit = 0;   // pixels that row tap r reaches
          for (int j = 0; j < MAX_BPT; ++j)
            if (ir[j] < na[j] && r == nr[j]) {
              rowhit |= 1u << j;
              nr[j] += g.sh;
              ++ir[j];
            }
          if (rowhit == 0) continue;
          int ns[MAX_BPT], is[MAX_BPT];
          for (int j = 0; j < MAX_BPT; ++j) { ns[j] = fs[j]; is[j] = 0; }
          for (int sx = 0; sx < g.S; ++sx) {
            bool any = false;
            for (int j = 0; j < MAX_BPT; ++j)
              if (is[j] < nb[j] && sx == ns[j]) {
                any |= (rowhit >> j) & 1u;
                ns[j] += g.sw;
                ++is[j];
              }
            taps += any;
          }
        }
      }
    }
    const int len = (taps > 1 ? taps : 1) * nkc;
    t.pre[ct + 1] = len;
    sum += len;
  }
  t.part[tid] = sum;
}

// Phase 8 (after part[] has become its inclusive running sum): lengths -> starts.
template <class P>
CS_PO_FN void phase_prefix(const Tables<P>& t, int CT, int tid, int T) {
  int t0, t1;
  tile_stretch(CT, tid, T, t0, t1);
  int run = tid > 0 ? t.part[tid - 1] : 0;
  for (int ct = t0; ct < t1; ++ct) {
    run += t.pre[ct + 1];
    t.pre[ct + 1] = run;
  }
  if (tid == 0) t.pre[0] = 0;
}

}  // namespace po
}  // namespace cs
