/*
 * conv_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, direct-loop CPU definition of what one device computes for its
 * share of a convolutional layer in arXiv 1712.02546: every device gets the
 * same input maps and a contiguous block [k0,k1) of the layer's kernels
 * (Section 4.1.2, Algorithms 1 and 2: "for maps = 1..numMaps: output =
 * convn(inputs, maps)"), and the abstract counts the backward convolutions in
 * the distributed work as well.  The paper prints no convolution formula, so
 * the three functions are the textbook definitions:
 *
 *   forward      y[n,k,p,q]  = sum_{c,r,s} x[n,c,p*sh-ph+r,q*sw-pw+s] * w[k,c,r,s]
 *   input grad   dx = d<y,dy>/dx   (sum over the kernels of the slice only)
 *   weight grad  dw = d<y,dy>/dw   (rows k0..k1-1 only)
 *
 * with x = 0 outside the image, cross-correlation (no kernel flip; MATLAB's
 * convn flips, which is only a relabelling of w), no bias, no activation.
 * P = floor((H+2ph-R)/sh)+1, Q likewise.  Layouts are row-major NCHW / KCRS
 * (the paper's extents in, inCh, k, numK, out, batch of Eq. (2), re-ordered).
 *
 * Everything is double: inputs, accumulators, outputs.  No blocking, no
 * im2col, no BLAS; OpenMP only over outputs that do not interact.  Tensors
 * y, dy, w, dw are FULL-layer tensors (K channels); a call reads/writes only
 * channels k0..k1-1 and leaves the rest of y / dw untouched.
 *
 * Nothing here is shared with the HIP path.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may load this file's library.
 *
 * Pins (tests/test_oracle_pins.py): exact finite differences (the loss is
 * bilinear), adjoint identities, slice concatenation / summation, 1x1 = matrix
 * product, full-size filter = dot product, one-hot filter = shift, all-ones =
 * tap count, unread trailing rows, and an independent library cross-check.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

typedef struct {
  int32_t N, C, H, W;      /* input  x[N][C][H][W]               */
  int32_t K, R, S;         /* filter w[K][C][R][S], full layer   */
  int32_t sh, sw, ph, pw;  /* stride and zero padding            */
  int32_t k0, k1;          /* this device's kernels              */
} oracle_shape_t;

static int out_extent(int in, int pad, int flt, int stride) {
  int span = in + 2 * pad - flt;
  if (span < 0) return 0;
  return span / stride + 1;
}

static int shape_ok(const oracle_shape_t *g) {
  if (!g) return 0;
  if (g->N < 1 || g->C < 1 || g->H < 1 || g->W < 1) return 0;
  if (g->K < 1 || g->R < 1 || g->S < 1) return 0;
  if (g->sh < 1 || g->sw < 1 || g->ph < 0 || g->pw < 0) return 0;
  if (g->k0 < 0 || g->k1 > g->K || g->k0 > g->k1) return 0;
  if (out_extent(g->H, g->ph, g->R, g->sh) < 1) return 0;
  if (out_extent(g->W, g->pw, g->S, g->sw) < 1) return 0;
  return 1;
}

int oracle_out_hw(const oracle_shape_t *g, int32_t *P, int32_t *Q) {
  if (!shape_ok(g)) return -1;
  *P = out_extent(g->H, g->ph, g->R, g->sh);
  *Q = out_extent(g->W, g->pw, g->S, g->sw);
  return 0;
}

/* Forward pass, Algorithm 2's convolution loop over the device's own maps. */
int oracle_conv_fwd(const oracle_shape_t *g, const double *x, const double *w,
                    double *y) {
  if (!shape_ok(g) || !x || !w || !y) return -1;
  const int P = out_extent(g->H, g->ph, g->R, g->sh);
  const int Q = out_extent(g->W, g->pw, g->S, g->sw);
  const int64_t C = g->C, H = g->H, W = g->W, K = g->K, R = g->R, S = g->S;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < g->N; ++n)
    for (int k = g->k0; k < g->k1; ++k)
      for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
          double acc = 0.0;
          for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r) {
              const int h = p * g->sh - g->ph + r;
              if (h < 0 || h >= H) continue;
              for (int s = 0; s < S; ++s) {
                const int v = q * g->sw - g->pw + s;
                if (v < 0 || v >= W) continue;
                acc += x[((n * C + c) * H + h) * W + v] *
                       w[((k * C + c) * R + r) * S + s];
              }
            }
          y[((n * K + k) * P + p) * Q + q] = acc;
        }
  return 0;
}

/*
 * Input gradient.  <y,dy> = sum_{n,k,p,q} dy * sum_{c,r,s} x*w, so every
 * product x[n,c,h,v]*w[k,c,r,s] that enters y[n,k,p,q] sends dy[n,k,p,q] *
 * w[k,c,r,s] to dx[n,c,h,v]: the forward loops with the roles of x and the
 * result swapped.  Only kernels of the slice contribute (a partial sum when
 * the slice is not the whole layer).  dx is overwritten.
 */
int oracle_conv_bwd_data(const oracle_shape_t *g, const double *dy,
                         const double *w, double *dx) {
  if (!shape_ok(g) || !dy || !w || !dx) return -1;
  const int P = out_extent(g->H, g->ph, g->R, g->sh);
  const int Q = out_extent(g->W, g->pw, g->S, g->sw);
  const int64_t C = g->C, H = g->H, W = g->W, K = g->K, R = g->R, S = g->S;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < g->N; ++n) {
    double *dxn = dx + n * C * H * W;
    memset(dxn, 0, sizeof(double) * (size_t)(C * H * W));
    for (int k = g->k0; k < g->k1; ++k)
      for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
          const double up = dy[((n * K + k) * P + p) * Q + q];
          for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r) {
              const int h = p * g->sh - g->ph + r;
              if (h < 0 || h >= H) continue;
              for (int s = 0; s < S; ++s) {
                const int v = q * g->sw - g->pw + s;
                if (v < 0 || v >= W) continue;
                dxn[(c * H + h) * W + v] += up * w[((k * C + c) * R + r) * S + s];
              }
            }
        }
  }
  return 0;
}

/* Weight gradient: the same products, collected per filter tap. */
int oracle_conv_bwd_weight(const oracle_shape_t *g, const double *x,
                           const double *dy, double *dw) {
  if (!shape_ok(g) || !x || !dy || !dw) return -1;
  const int P = out_extent(g->H, g->ph, g->R, g->sh);
  const int Q = out_extent(g->W, g->pw, g->S, g->sw);
  const int64_t C = g->C, H = g->H, W = g->W, K = g->K, R = g->R, S = g->S;
#pragma omp parallel for collapse(2) schedule(static)
  for (int k = g->k0; k < g->k1; ++k)
    for (int c = 0; c < g->C; ++c)
      for (int r = 0; r < R; ++r)
        for (int s = 0; s < S; ++s) {
          double acc = 0.0;
          for (int n = 0; n < g->N; ++n)
            for (int p = 0; p < P; ++p) {
              const int h = p * g->sh - g->ph + r;
              if (h < 0 || h >= H) continue;
              for (int q = 0; q < Q; ++q) {
                const int v = q * g->sw - g->pw + s;
                if (v < 0 || v >= W) continue;
                acc += dy[((n * K + k) * P + p) * Q + q] *
                       x[((n * C + c) * H + h) * W + v];
              }
            }
          dw[((k * C + c) * R + r) * S + s] = acc;
        }
  return 0;
}

/*
 * Single-element versions for spot checks at sizes where the full loops take
 * minutes.  idx[] holds flat row-major indices into y / dx / dw; out[i] is
 * that element.  The input-gradient one is written the other way round from
 * the full version (it looks for the windows that cover a pixel), so the two
 * check each other.
 */
int oracle_conv_fwd_at(const oracle_shape_t *g, const double *x,
                       const double *w, const int64_t *idx, int64_t count,
                       double *out) {
  if (!shape_ok(g) || !x || !w || !idx || !out || count < 0) return -1;
  const int P = out_extent(g->H, g->ph, g->R, g->sh);
  const int Q = out_extent(g->W, g->pw, g->S, g->sw);
  const int64_t C = g->C, H = g->H, W = g->W, K = g->K, R = g->R, S = g->S;
  const int64_t total = (int64_t)g->N * K * P * Q;
  for (int64_t i = 0; i < count; ++i)
    if (idx[i] < 0 || idx[i] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t i = 0; i < count; ++i) {
    int64_t t = idx[i];
    const int q = (int)(t % Q); t /= Q;
    const int p = (int)(t % P); t /= P;
    const int64_t k = t % K;
    const int64_t n = t / K;
    double acc = 0.0;
    if (k >= g->k0 && k < g->k1)
      for (int c = 0; c < C; ++c)
        for (int r = 0; r < R; ++r) {
          const int h = p * g->sh - g->ph + r;
          if (h < 0 || h >= H) continue;
          for (int s = 0; s < S; ++s) {
            const int v = q * g->sw - g->pw + s;
            if (v < 0 || v >= W) continue;
            acc += x[((n * C + c) * H + h) * W + v] *
                   w[((k * C + c) * R + r) * S + s];
          }
        }
    out[i] = acc;
  }
  return 0;
}

int oracle_conv_bwd_data_at(const oracle_shape_t *g, const double *dy,
                            const double *w, const int64_t *idx, int64_t count,
                            double *out) {
  if (!shape_ok(g) || !dy || !w || !idx || !out || count < 0) return -1;
  const int P = out_extent(g->H, g->ph, g->R, g->sh);
  const int Q = out_extent(g->W, g->pw, g->S, g->sw);
  const int64_t C = g->C, H = g->H, W = g->W, K = g->K, R = g->R, S = g->S;
  const int64_t total = (int64_t)g->N * C * H * W;
  for (int64_t i = 0; i < count; ++i)
    if (idx[i] < 0 || idx[i] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t i = 0; i < count; ++i) {
    int64_t t = idx[i];
    const int v = (int)(t % W); t /= W;
    const int h = (int)(t % H); t /= H;
    const int64_t c = t % C;
    const int64_t n = t / C;
    double acc = 0.0;
    for (int64_t k = g->k0; k < g->k1; ++k)
      for (int r = 0; r < R; ++r) {
        const int hh = h + g->ph - r;           /* = p*sh for a covering window */
        if (hh < 0 || hh % g->sh) continue;
        const int p = hh / g->sh;
        if (p >= P) continue;
        for (int s = 0; s < S; ++s) {
          const int vv = v + g->pw - s;
          if (vv < 0 || vv % g->sw) continue;
          const int q = vv / g->sw;
          if (q >= Q) continue;
          acc += dy[((n * K + k) * P + p) * Q + q] *
                 w[((k * C + c) * R + r) * S + s];
        }
      }
    out[i] = acc;
  }
  return 0;
}

int oracle_conv_bwd_weight_at(const oracle_shape_t *g, const double *x,
                              const double *dy, const int64_t *idx,
                              int64_t count, double *out) {
  if (!shape_ok(g) || !x || !dy || !idx || !out || count < 0) return -1;
  const int P = out_extent(g->H, g->ph, g->R, g->sh);
  const int Q = out_extent(g->W, g->pw, g->S, g->sw);
  const int64_t C = g->C, H = g->H, W = g->W, K = g->K, R = g->R, S = g->S;
  const int64_t total = K * C * R * S;
  for (int64_t i = 0; i < count; ++i)
    if (idx[i] < 0 || idx[i] >= total) return -2;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t i = 0; i < count; ++i) {
    int64_t t = idx[i];
    const int s = (int)(t % S); t /= S;
    const int r = (int)(t % R); t /= R;
    const int64_t c = t % C;
    const int64_t k = t / C;
    double acc = 0.0;
    if (k >= g->k0 && k < g->k1)
      for (int64_t n = 0; n < g->N; ++n)
        for (int p = 0; p < P; ++p) {
          const int h = p * g->sh - g->ph + r;
          if (h < 0 || h >= H) continue;
          for (int q = 0; q < Q; ++q) {
            const int v = q * g->sw - g->pw + s;
            if (v < 0 || v >= W) continue;
            acc += dy[((n * K + k) * P + p) * Q + q] *
                   x[((n * C + c) * H + h) * W + v];
          }
        }
    out[i] = acc;
  }
  return 0;
}

#ifdef _OPENMP
#include <omp.h>
int oracle_threads(void) { return omp_get_max_threads(); }
#else
int oracle_threads(void) { return 1; }
#endif
