/*
 * Driver for a sanitizer build of the CPU oracle (oracle/conv_oracle.c): every
 * routine runs on exactly sized heap arrays, so AddressSanitizer sees any read
 * or write outside a tensor and UndefinedBehaviorSanitizer any overflow or bad
 * shift in the index arithmetic.  Results are also checked against what the
 * mathematics fixes: the adjoint identities <conv(x,w),dy> = <x,dx> = <w,dw>
 * and the element-wise routines against the full loops.
 *
 * Build: gcc -std=c11 -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp
 *            oracle/conv_oracle.c tests/oracle_sanitize_main.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct {
  int32_t N, C, H, W, K, R, S, sh, sw, ph, pw, k0, k1;
} shape_t;

int oracle_out_hw(const shape_t *g, int32_t *P, int32_t *Q);
int oracle_conv_fwd(const shape_t *g, const double *x, const double *w, double *y);
int oracle_conv_bwd_data(const shape_t *g, const double *dy, const double *w, double *dx);
int oracle_conv_bwd_weight(const shape_t *g, const double *x, const double *dy, double *dw);
int oracle_conv_fwd_at(const shape_t *g, const double *x, const double *w, const int64_t *idx, int64_t n, double *out);
int oracle_conv_bwd_data_at(const shape_t *g, const double *dy, const double *w, const int64_t *idx, int64_t n, double *out);
int oracle_conv_bwd_weight_at(const shape_t *g, const double *x, const double *dy, const int64_t *idx, int64_t n, double *out);

static uint64_t lcg = 88172645463325252ull;
static double rnd(void) {
  lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
  return (double)(int64_t)(lcg >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static double *filled(int64_t n) {
  double *p = malloc(sizeof(double) * (size_t)n);
  for (int64_t i = 0; i < n; ++i) p[i] = rnd();
  return p;
}
static double dot(const double *a, const double *b, int64_t n) {
  double s = 0;
  for (int64_t i = 0; i < n; ++i) s += a[i] * b[i];
  return s;
}
static int close_to(double a, double b, double scale) { return fabs(a - b) <= 1e-11 * (fabs(scale) + 1.0); }

static int run(shape_t g) {
  int32_t P, Q;
  if (oracle_out_hw(&g, &P, &Q) != 0) return 0; /* not a valid shape: nothing to check */
  const int64_t nx = (int64_t)g.N * g.C * g.H * g.W, nw = (int64_t)g.K * g.C * g.R * g.S;
  const int64_t ny = (int64_t)g.N * g.K * P * Q;
  double *x = filled(nx), *w = filled(nw), *dy = filled(ny);
  double *y = calloc((size_t)ny, sizeof(double)), *dx = filled(nx), *dw = calloc((size_t)nw, sizeof(double));
  int bad = 0;
  bad |= oracle_conv_fwd(&g, x, w, y) != 0;
  bad |= oracle_conv_bwd_data(&g, dy, w, dx) != 0;
  bad |= oracle_conv_bwd_weight(&g, x, dy, dw) != 0;
  /* kernels outside the slice give no y and no dw, so the three inner products agree for any slice */
  const double a = dot(y, dy, ny), b = dot(x, dx, nx), c = dot(w, dw, nw);
  if (!close_to(a, b, a) || !close_to(a, c, a)) {
    fprintf(stderr, "adjoint identities: %.15g %.15g %.15g\n", a, b, c);
    bad = 1;
  }
  const int64_t most = nx > ny ? (nx > nw ? nx : nw) : (ny > nw ? ny : nw);
  int64_t *idx = malloc(sizeof(int64_t) * (size_t)most);
  double *out = malloc(sizeof(double) * (size_t)most);
  for (int64_t i = 0; i < most; ++i) idx[i] = i;
  bad |= oracle_conv_fwd_at(&g, x, w, idx, ny, out) != 0;
  for (int64_t i = 0; i < ny && !bad; ++i) bad |= !close_to(out[i], y[i], y[i]);
  bad |= oracle_conv_bwd_data_at(&g, dy, w, idx, nx, out) != 0;
  for (int64_t i = 0; i < nx && !bad; ++i) bad |= !close_to(out[i], dx[i], dx[i]);
  bad |= oracle_conv_bwd_weight_at(&g, x, dy, idx, nw, out) != 0;
  for (int64_t i = 0; i < nw && !bad; ++i) bad |= !close_to(out[i], dw[i], dw[i]);
  /* an index one past the end must be refused, not read */
  idx[0] = ny;
  bad |= oracle_conv_fwd_at(&g, x, w, idx, 1, out) == 0;
  if (bad)
    fprintf(stderr, "FAILED N%d C%d H%d W%d K%d R%d S%d stride %d,%d pad %d,%d slice [%d,%d)\n", g.N, g.C, g.H, g.W,
            g.K, g.R, g.S, g.sh, g.sw, g.ph, g.pw, g.k0, g.k1);
  free(x); free(w); free(dy); free(y); free(dx); free(dw); free(idx); free(out);
  return bad;
}

int main(void) {
  int bad = 0, cases = 0;
  for (int R = 1; R <= 5; R += 2)
    for (int S = 1; S <= 4; ++S)
      for (int sh = 1; sh <= 3; ++sh)
        for (int sw = 1; sw <= 3; sw += 2)
          for (int ph = 0; ph <= 2; ++ph)
            for (int pw = 0; pw <= 3; pw += 3) {
              shape_t g = {2, 3, 6 + R % 3, 5 + S, 4, R, S, sh, sw, ph, pw, (R + S) % 3, 4 - (ph & 1)};
              bad |= run(g);
              ++cases;
            }
  /* unread trailing rows, a one-element problem, P = Q = 1, an empty slice */
  bad |= run((shape_t){1, 1, 34, 34, 1, 5, 5, 4, 4, 0, 0, 0, 1});
  bad |= run((shape_t){1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 0, 1});
  bad |= run((shape_t){3, 2, 6, 6, 5, 6, 6, 1, 1, 0, 0, 1, 4});
  bad |= run((shape_t){2, 2, 5, 5, 3, 3, 3, 1, 1, 1, 1, 2, 2});
  printf("%s %d cases\n", bad ? "FAILED" : "ok", cases + 4);
  return bad;
}
