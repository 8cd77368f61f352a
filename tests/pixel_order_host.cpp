// Host build of the input-gradient pixel ordering (csrc/pixel_order.h): the phases the GPU
// kernel runs, executed thread after thread on tables whose every access is bounds-checked
// against the extents the kernel declares.  Checks, for each geometry on the command line or
// in the built-in sweep: no access outside a table; perm is a permutation of the pixels;
// tap counts do not increase along it; pixels with the same set of taps are neighbours; pre
// starts at 0, and pre[ct+1]-pre[ct] is nkc * max(1, taps reaching any pixel of tile ct),
// counted here by brute force, for column tiles of four and of eight blocks.
//
// Build: g++ -std=c++17 -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all
#include <cstdio>
#include <cstdlib>
#include <set>
#include <vector>

struct Checked {
  int* p;
  int n;
  const char* name;
  int& operator[](long i) const {
    if (i < 0 || i >= n) {
      std::fprintf(stderr, "OUT OF BOUNDS: %s[%ld], extent %d\n", name, i, n);
      std::abort();
    }
    return p[i];
  }
};
Checked view(const Checked& b, int off, int len) {
  if (off < 0 || len < 0 || off + len > b.n) {
    std::fprintf(stderr, "OUT OF BOUNDS: view [%d,%d) of %s, extent %d\n", off, off + len, b.name, b.n);
    std::abort();
  }
  return Checked{b.p + off, len, b.name};
}

#include "../paper_1712_02546_amd/csrc/pixel_order.h"

namespace po = cs::po;

static int out_extent(int in, int pad, int flt, int stride) {
  const long span = (long)in + 2L * pad - flt;
  return span < 0 ? 0 : (int)(span / stride) + 1;
}

struct Case {
  int H, W, R, S, sh, sw, ph, pw, NB, nkc, T;
};

static long g_cases = 0;

#define FAIL(...)                                                                                        \
  do {                                                                                                   \
    std::fprintf(stderr, "FAIL H=%d W=%d R=%d S=%d stride=%d,%d pad=%d,%d NB=%d nkc=%d T=%d: ", c.H, c.W, \
                 c.R, c.S, c.sh, c.sw, c.ph, c.pw, c.NB, c.nkc, c.T);                                    \
    std::fprintf(stderr, __VA_ARGS__);                                                                   \
    std::fprintf(stderr, "\n");                                                                          \
    return false;                                                                                        \
  } while (0)

static bool run_case(const Case& c, int bpt);
static bool run_case(const Case& c) { return run_case(c, 4) && run_case(c, 8); }

static bool run_case(const Case& c, int bpt) {
  cs::Geo g{};
  g.H = c.H; g.W = c.W; g.R = c.R; g.S = c.S; g.sh = c.sh; g.sw = c.sw; g.ph = c.ph; g.pw = c.pw;
  g.P = out_extent(c.H, c.ph, c.R, c.sh);
  g.Q = out_extent(c.W, c.pw, c.S, c.sw);
  if (g.P < 1 || g.Q < 1 || (long)c.R * c.S > po::MAX_RS) return true;   // not a shape the library admits
  g.NB = c.NB; g.Np = 32 * c.NB; g.N = g.Np;
  g.HW = c.H * c.W; g.PQ = g.P * g.Q; g.RS = c.R * c.S;
  ++g_cases;
  const int CT = (g.HW * g.NB + bpt - 1) / bpt;
  // extents exactly as the kernel declares them (static LDS arrays) or the host plan allocates them
  std::vector<int> bins(po::BINS, -1), rowCnt(po::AXIS_CNT, -1), colCnt(po::AXIS_CNT, -1), part(c.T, -1);
  const bool in_lds = po::axes_ints(g.H, g.W) <= po::AXES_LDS;
  std::vector<int> axes(in_lds ? po::AXES_LDS : po::axes_ints(g.H, g.W), -1);
  std::vector<int> perm(g.HW, -1), pre(CT + 2, -1);
  po::Tables<Checked> t;
  t.bins = Checked{bins.data(), (int)bins.size(), "bins"};
  t.rowCnt = Checked{rowCnt.data(), (int)rowCnt.size(), "rowCnt"};
  t.colCnt = Checked{colCnt.data(), (int)colCnt.size(), "colCnt"};
  t.part = Checked{part.data(), (int)part.size(), "part"};
  t.axes = Checked{axes.data(), (int)axes.size(), "axes"};
  t.perm = Checked{perm.data(), (int)perm.size(), "perm"};
  t.pre = Checked{pre.data(), (int)pre.size(), "pre"};
  const int T = c.T;
  for (int tid = 0; tid < T; ++tid) po::phase_axes(g, t, tid, T);
  for (int tid = 0; tid < T; ++tid) po::phase_ranks(g, t, tid, T);
  for (int tid = 0; tid < T; ++tid) po::phase_bins(g, t, tid, T);
  for (int tid = 0; tid < T; ++tid) po::phase_scan_bins(g, t, tid, T);
  for (int tid = 0; tid < T; ++tid) po::phase_place(g, t, tid, T);
  for (int tid = 0; tid < T; ++tid) po::phase_lengths(g, t, CT, c.nkc, bpt, tid, T);
  for (int tid = 1; tid < T; ++tid) part[tid] += part[tid - 1];   // the kernel's workgroup scan
  for (int tid = 0; tid < T; ++tid) po::phase_prefix(t, CT, tid, T);

  // --- the reference view: which taps reach a pixel, by the definition ---
  auto reaches = [&](int px, int r, int s) {
    const int hr = px / g.W + g.ph - r, vs = px % g.W + g.pw - s;
    return hr >= 0 && vs >= 0 && hr % g.sh == 0 && vs % g.sw == 0 && hr / g.sh < g.P && vs / g.sw < g.Q;
  };
  std::vector<int> taps(g.HW, 0);
  std::vector<std::vector<int>> tapset(g.HW);
  for (int px = 0; px < g.HW; ++px)
    for (int r = 0; r < g.R; ++r)
      for (int s = 0; s < g.S; ++s)
        if (reaches(px, r, s)) {
          ++taps[px];
          tapset[px].push_back(r * g.S + s);
        }
  std::vector<char> seen(g.HW, 0);
  for (int i = 0; i < g.HW; ++i) {
    const int px = perm[i];
    if (px < 0 || px >= g.HW) FAIL("perm[%d] = %d is no pixel", i, px);
    if (seen[px]) FAIL("pixel %d placed twice", px);
    seen[px] = 1;
    if (i > 0 && taps[perm[i - 1]] < taps[px]) FAIL("tap count rises at position %d", i);
  }
  std::set<std::vector<int>> closed;   // tap sets whose group has ended
  for (int i = 0; i < g.HW; ++i) {
    if (i > 0 && tapset[perm[i]] != tapset[perm[i - 1]]) closed.insert(tapset[perm[i - 1]]);
    if (closed.count(tapset[perm[i]])) FAIL("pixels with one tap set are not contiguous (position %d)", i);
  }
  if (pre[0] != 0) FAIL("pre[0] = %d", pre[0]);
  for (int ct = 0; ct < CT; ++ct) {
    std::set<int> u;
    for (int j = 0; j < bpt; ++j) {
      const int gcb = ct * bpt + j;
      if (gcb >= g.HW * g.NB) break;
      for (int tp : tapset[perm[gcb / g.NB]]) u.insert(tp);
    }
    const int want = c.nkc * (u.empty() ? 1 : (int)u.size());
    if (pre[ct + 1] - pre[ct] != want)
      FAIL("tile %d of %d blocks: length %d, expected %d", ct, bpt, pre[ct + 1] - pre[ct], want);
  }
  if (pre[CT + 1] != -1) FAIL("pre written past CT");
  return true;
}

int main(int argc, char** argv) {
  if (argc == 12) {   // one geometry from the command line
    Case c{std::atoi(argv[1]), std::atoi(argv[2]), std::atoi(argv[3]), std::atoi(argv[4]), std::atoi(argv[5]),
           std::atoi(argv[6]), std::atoi(argv[7]), std::atoi(argv[8]), std::atoi(argv[9]), std::atoi(argv[10]),
           std::atoi(argv[11])};
    if (!run_case(c)) return 1;
    std::printf("ok 1 case\n");
    return 0;
  }
  const int mode = argc > 1 ? std::atoi(argv[1]) : 0;
  bool ok = true;
  if (mode == 0) {
    // small filter extents, the extents on both sides of 32, long ones; strides 1-4, pads 0-3
    const int F[] = {1, 2, 3, 4, 5, 7, 8, 11, 12, 31, 32, 33, 34, 64, 100};
    for (int R : F)
      for (int S : F) {
        if (R * S > po::MAX_RS) continue;
        for (int st = 1; st <= 4; ++st)
          for (int pad = 0; pad <= 3; ++pad) {
            const int H = R + 3 + (R * 7 + st) % 5, W = S + 2 + (S * 5 + pad) % 6;
            const int NB = 1 + (R + S + st + pad) % 4;
            ok &= run_case(Case{H, W, R, S, st, st, pad, pad, NB, 1 + (R + pad) % 3, 1024});
          }
      }
    // rectangular strides and pads, thread counts other than the kernel's
    for (int sh = 1; sh <= 4; ++sh)
      for (int sw = 1; sw <= 4; ++sw)
        for (int ph = 0; ph <= 3; ++ph)
          for (int pw = 0; pw <= 3; ++pw) {
            ok &= run_case(Case{23, 19, 7, 4, sh, sw, ph, pw, 3, 2, 64});
            ok &= run_case(Case{40, 10, 33, 3, sh, sw, ph, pw, 1, 1, 1024});
          }
  } else {
    // the long and thin limits: R or S up to 1024, images with more rows than the LDS tables hold
    for (int R : {128, 255, 256, 512, 1000, 1024})
      for (int st : {1, 2, 3, 4})
        for (int pad : {0, 1, 3}) {
          ok &= run_case(Case{R + 6, 3, R, 1, st, st, pad, pad, 1, 1, 1024});
          ok &= run_case(Case{3, R + 6, 1, R, st, st, pad, pad, 2, 2, 1024});
          if (R <= 512) ok &= run_case(Case{R + 9, 5, R, 2, st, st, pad, pad, 1, 1, 1024});
        }
    ok &= run_case(Case{1100, 40, 5, 5, 1, 1, 2, 2, 1, 3, 1024});   // 6H + 5W > the LDS table: global scratch extents
    ok &= run_case(Case{30, 1300, 3, 3, 2, 2, 1, 1, 1, 1, 1024});
    ok &= run_case(Case{14, 14, 5, 5, 1, 1, 0, 0, 4, 47, 1024});    // the 1500-kernel layer
    ok &= run_case(Case{224, 224, 11, 11, 4, 4, 2, 2, 2, 3, 1024});
  }
  std::printf("%s %ld cases\n", ok ? "ok" : "FAILED", g_cases);
  return ok ? 0 : 1;
}
