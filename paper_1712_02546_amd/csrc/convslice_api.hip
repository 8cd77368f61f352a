// Host side of libconvslice.so: argument checks, workspace carving and kernel
// launches for the three passes declared in include/convslice.h.
#include "../../include/convslice.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>
#include <type_traits>
#include <vector>

#include "conv_common.h"
#include "conv_internal.h"
#include "gemm_kernels.h"
#include "gemm_bf16_kernels.h"
#include "pack_kernels.h"
#include "pm_kernels.h"

namespace {

using cs::Geo;

// Work copies are addressed with 32-bit byte offsets from a base a little in front of them.
constexpr int64_t kMaxElems = ((int64_t)1 << 30) - 4096;

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

int out_extent(int in, int pad, int flt, int stride) {
  const int64_t span = (int64_t)in + 2 * (int64_t)pad - flt;
  if (span < 0) return 0;
  return (int)(span / stride) + 1;
}

// Validates the descriptor and derives the geometry.  No GPU call.
int make_geo(const conv_desc_t* d, Geo& g) {
  if (!d) return CONV_ERR_NULL;
  if (d->dtype != CONV_F32 && d->dtype != CONV_BF16) return CONV_ERR_DTYPE;
  if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->R < 1 || d->S < 1)
    return CONV_ERR_SHAPE;
  if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0) return CONV_ERR_SHAPE;
  if (d->k0 < 0 || d->k1 > d->K || d->k0 > d->k1) return CONV_ERR_SLICE;
  const int P = out_extent(d->H, d->pad_h, d->R, d->stride_h);
  const int Q = out_extent(d->W, d->pad_w, d->S, d->stride_w);
  if (P < 1 || Q < 1) return CONV_ERR_SHAPE;
  if ((int64_t)d->R * d->S > cs::po::MAX_RS) return CONV_ERR_SHAPE;
  if (d->pad_h > (1 << 20) || d->pad_w > (1 << 20)) return CONV_ERR_SHAPE;
  const int64_t Np = round_up(d->N, 32);
  const int64_t HW = (int64_t)d->H * d->W, PQ = (int64_t)P * Q, RS = (int64_t)d->R * d->S;
  const int64_t Cp = round_up(d->C, 4);
  if ((int64_t)d->C * HW * Np >= kMaxElems) return CONV_ERR_SHAPE;       // x, x_t, dx_t
  if (((int64_t)d->K + 32) * (PQ + 1) * Np >= kMaxElems) return CONV_ERR_SHAPE;   // y, dy and work copies (padded)
  if (((int64_t)PQ + 1) * Np >= ((int64_t)1 << 29)) return CONV_ERR_SHAPE;          // two rows of a work copy in 32 bits
  // w and its work copies: rows re-pitched to a multiple of 32 (fwd), kernels padded to a multiple of 32 (bwd_data)
  if ((int64_t)d->K * (round_up(Cp * RS, 32) + 32) >= kMaxElems) return CONV_ERR_SHAPE;
  if (((int64_t)d->K + 32) * Cp * RS >= kMaxElems) return CONV_ERR_SHAPE;
  g.N = d->N; g.Np = (int)Np; g.NB = (int)(Np / 32);
  g.C = d->C; g.H = d->H; g.W = d->W; g.K = d->K; g.R = d->R; g.S = d->S; g.P = P; g.Q = Q;
  g.sh = d->stride_h; g.sw = d->stride_w; g.ph = d->pad_h; g.pw = d->pad_w;
  g.k0 = d->k0; g.Ks = d->k1 - d->k0;
  g.HW = (int)HW; g.PQ = (int)PQ; g.RS = (int)RS; g.CRS = (int)(d->C * RS);
  return CONV_OK;
}

inline size_t seg(int64_t floats) { return (size_t)round_up(floats * 4, 256); }
// A buffer that the DMA loaders read gets a zero page directly in front of it.
constexpr size_t kZeroBytes = cs::ZERO_PAGE_FLOATS * 4;

// Workgroup slots on the chip: two 64 KB workgroups fit a compute unit's 160 KB of LDS.
int chip_slots() {
  static int slots = 0;
  if (slots == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      slots = 2 * cus;
    else
      return 512;   // no device visible (workspace queries on a CPU-only host): MI355X has 256 CUs
  }
  return slots;
}

// Splits T equal tiles of nch chunks into whole-tile rounds and an evenly shared tail.
// share_cost: what sharing a tail costs (scratch round trip of the cut tiles, fix-up launch), in chunk times; the
// tail is shared only if the idle slots it fills are worth more: nch * (S - rem) / S chunk times.
cs::TailPlan plan_tail(int T, int nch, int S = 0, int share_cost = 0) {
  cs::TailPlan tp;
  if (S <= 0) S = chip_slots();
  const int rem = T % S;
  // nothing left over, reductions too short to be worth splitting, or too few idle slots to pay for the sharing
  if (rem == 0 || nch < 16 || (int64_t)nch * (S - rem) < (int64_t)share_cost * S) {
    tp.nFull = T; tp.nTail = 0; tp.units = 1; tp.nTailWg = 0;
    return tp;
  }
  tp.nFull = T - rem;
  tp.nTail = rem;
  const int64_t work = (int64_t)rem * nch;
  // Equal runs over all slots, but no tile in more than 16 pieces: the fix-up kernel adds a tile's slots one after
  // the other, and a handful of tail tiles cut 500 ways would cost more there than they save here.
  tp.units = (int)std::max<int64_t>((work + S - 1) / S, (nch + 15) / 16);
  tp.nTailWg = (int)((work + tp.units - 1) / tp.units);
  return tp;
}
// Scratch slots for a shared tail: the most any slice of the layer can need (two per workgroup slot), so that the
// workspace size does not depend on how the tile count of a slice happens to divide.
inline size_t tail_bytes(int nch) {
  return nch >= 16 ? (size_t)chip_slots() * 2 * cs::TAIL_SLOT_FLOATS * 4 : 0;
}

// Row tiles of a matrix-core pass with M rows: `full` tiles of 128 rows and, when the rest is at most 64 rows, one
// half tile (64 rows) for it, computed by a second launch; a rest above 64 rows takes a full tile -- or, where the
// pass has the 96-row kernels (three_quarter), a rest of 65..96 rows takes a 96-row tile.
// When 96-row tiles alone cover M in no more rows than that mix, they are used for the whole pass: one launch
// instead of two (a 188-kernel share: two 96-row tiles instead of 128 + 64).
struct RowSplit {
  int full, half;   // half = 1 if a half tile follows the full ones
  int last;         // shape (cs::Shape) of the launch after the full tiles: 0 none, 1: 64 rows, 3: 96 rows
  int nlast;        // its row tiles
};
RowSplit split_rows(int M, bool three_quarter = false) {
  RowSplit r;
  r.full = M / cs::BM;
  const int rest = M - r.full * cs::BM;
  r.half = rest > 0 && rest <= cs::BM / 2;
  r.last = r.half ? 1 : 0;
  r.nlast = r.half ? 1 : 0;
  if (rest > cs::BM / 2) {
    if (three_quarter && rest <= 96) { r.last = 3; r.nlast = 1; }
    else ++r.full;
  }
  if (three_quarter && r.full > 0 && r.last != 0) {
    const int rows = r.full * cs::BM + (r.last == 1 ? 64 : 96), n96 = (M + 95) / 96;
    // (no more row tiles than 128-row tiles would be: the split partials of the weight gradient are sized by those)
    if (n96 * 96 <= rows && n96 <= (M + cs::BM - 1) / cs::BM) { r.full = 0; r.half = 0; r.last = 3; r.nlast = n96; }
  }
  return r;
}

struct FwdPlan {
  bool repitch;      // filters copied to zero-padded fp32 rows of pitch ldw (bf16 input, or C*R*S not a multiple of BK)
  int ldw, nch;
  int CT;            // column tiles; the row tiles and tail plans are fixed per launch (launch_fwd_gemm)
  size_t off_xt, off_yt, off_w, off_tab, off_tail, total;
};

FwdPlan plan_fwd(const Geo& g, int dtype) {
  FwdPlan p;
  p.repitch = dtype != CONV_F32 || (g.CRS % cs::BK) != 0;
  p.ldw = p.repitch ? (int)round_up(g.CRS, cs::BK) : g.CRS;
  p.nch = (g.CRS + cs::BK - 1) / cs::BK;
  p.CT = (g.PQ * g.NB + 3) / 4;
  size_t o = 0;
  o += kZeroBytes;
  p.off_xt = o;  o += seg((int64_t)g.C * g.HW * g.Np);
  p.off_yt = o;  o += seg((int64_t)g.Ks * g.PQ * g.Np);
  p.off_w = o;   o += p.repitch ? seg((int64_t)g.Ks * p.ldw) : 0;
  p.off_tab = o; o += seg((int64_t)(p.nch + 4) * cs::BK * 2);
  p.off_tail = o; o += tail_bytes(p.nch);
  p.total = o;
  return p;
}

// Even sharing of the input-gradient pass: the line of column tiles is measured on the device (by the ordering
// kernel) and cut by the kernels themselves; the host only fixes the number of runs.  Each run of the line is
// computed by MB workgroups, one per row tile, which therefore walk through the same pixels, taps and k-chunks at
// the same time and share the dy operand.
// rounds: workgroups per slot.  One gives every workgroup the longest run; with three, a slot that is freed early
// (the two workgroups of a compute unit do not advance at the same pace) is refilled, which pays when the runs
// stay long.
inline int run_rounds(int64_t line, int MB) { return line / std::max(1, chip_slots() / MB) >= 250 ? 3 : 1; }
cs::RunPlan plan_runs(int MB, bool possible, int S = 0, int rounds = 1) {
  cs::RunPlan rp;
  rp.enabled = 0; rp.nRuns = 1; rp.nWg = 0;
  if (S <= 0) S = chip_slots();
  if (!possible || S / MB < 1) return rp;
  rp.enabled = 1;
  rp.nRuns = rounds * S / MB;
  rp.nWg = rp.nRuns * MB;
  return rp;
}

struct BwdDataPlan {
  bool scatter;   // few input channels: T = w^T * dy on the matrix cores, then a col2im gather
  int Cp, Ksp, nch, CT1;   // Ksp: pitch of w' in the scatter form, a multiple of BK; CT1: its column tiles
  int rounds;              // per-pixel form: workgroups per slot when the line is cut into runs (the most any launch uses)
  int64_t line;            // chunks on the line of column tiles, about
  size_t off_dyt, off_wt, off_dxt, off_perm, off_pre, off_scratch, off_tab, off_T, off_tail, total;
};

BwdDataPlan plan_bwd_data(const Geo& g) {
  BwdDataPlan p;
  p.Cp = (int)round_up(g.C, 4);
  p.Ksp = (int)round_up(g.Ks, cs::BK);
  p.nch = (g.Ks + cs::BK - 1) / cs::BK;
  // With C input channels the per-pixel form fills C of a tile's 128 rows; the scatter form
  // fills C*R*S of them and pays one round trip of T through memory instead.
  // Cost model (seconds up to a common factor): matrix-core time is the nominal work divided by the share of
  // tile rows that hold data; the scatter form adds one write and one read of T at HBM-side speed.  The choice
  // is made for the whole layer (K, not the slice), so that every slice of a layer takes the same form and a
  // workspace sized for a slice is large enough for any part of it.
  {
    const double F = 2.0 * g.Np * g.K * (double)g.CRS * g.PQ;
    auto tile_rows = [](int M) {   // rows the row tiles of an M-row pass compute
      const RowSplit r = split_rows(M, true);
      return r.full * cs::BM + (r.last == 1 ? 64 : r.last == 3 ? 96 : 0);
    };
    const double rows_pixel = (double)g.C / (double)tile_rows(g.C);
    const double rows_scatter = (double)g.CRS / (double)tile_rows(g.CRS);
    const double t_pixel = F / (130e12 * rows_pixel);
    const double t_scatter = F / (130e12 * rows_scatter) + 2.0 * 4.0 * g.CRS * (double)g.PQ * g.Np / 3e12;
    p.scatter = t_scatter < 0.9 * t_pixel && (int64_t)g.CRS * g.PQ * g.Np < kMaxElems;
  }
  size_t o = 0;
  if (p.scatter) {
    o += kZeroBytes;
    p.off_dyt = o;  o += seg((int64_t)g.Ks * g.PQ * g.Np);
    p.off_wt = o;   o += seg((int64_t)g.CRS * p.Ksp);          // w'[(c,r,s)][k], zero past Ks
    p.off_tab = o;  o += seg((int64_t)(p.nch + 4) * cs::BK * 2);
    p.off_T = o;    o += seg((int64_t)g.CRS * g.PQ * g.Np);
    p.CT1 = (g.PQ * g.NB + 3) / 4;
    p.off_tail = o; o += tail_bytes(p.nch);
    p.off_dxt = p.off_perm = 0;
    p.total = o;
    return p;
  }
  p.off_tab = p.off_T = 0;
  // dy_t[Ksp][PQ+1][Np] (one zero pixel per row, zero rows past Ks), w_t[RS][Ksp][Cp] (zero rows past Ks)
  p.off_dyt = o;  o += seg((int64_t)p.Ksp * (g.PQ + 1) * g.Np);
  p.off_wt = o;   o += seg((int64_t)g.RS * g.C * p.Ksp);
  p.off_dxt = o;  o += seg((int64_t)g.C * g.HW * g.Np);
  p.off_perm = o; o += seg(g.HW);
  const int CT = (g.HW * g.NB + 3) / 4;
  p.off_pre = o;  o += seg((int64_t)CT + 2);
  p.off_scratch = o; o += seg(cs::po::axes_ints(g.H, g.W));
  // Rounds of runs (plan_runs): three where a third of the line per slot is still a long run.  Chunks on the line,
  // about: taps that reach a pixel, summed over the pixels = (valid (p,r) pairs) x (valid (q,s) pairs), times the
  // column tiles per pixel and the k-chunks per tap.  (Measured: runs of 918 chunks 3.65 ms, three rounds of 306
  // 3.57 ms; 313 -> 104: 1.345 -> 1.307 ms; 131 -> 44: 0.597 -> 0.605 ms.)
  {
    int64_t rows = 0, cols = 0;
    for (int pp = 0; pp < g.P; ++pp)
      for (int r = 0; r < g.R; ++r) rows += (unsigned)(pp * g.sh - g.ph + r) < (unsigned)g.H;
    for (int q = 0; q < g.Q; ++q)
      for (int ss = 0; ss < g.S; ++ss) cols += (unsigned)(q * g.sw - g.pw + ss) < (unsigned)g.W;
    p.line = rows * cols * g.NB / 4 * p.nch;
    p.rounds = run_rounds(p.line, (g.C + cs::BM - 1) / cs::BM);
  }
  p.off_tail = o; o += (size_t)p.rounds * chip_slots() * 2 * cs::TAIL_SLOT_FLOATS * 4;   // two slots per workgroup
  p.total = o;
  return p;
}

// Number of pieces the weight gradient's reduction (nch chunks) is cut into when the output has `tiles` tiles.
// fp32 (the matrix pipe is the limit): cost model in chunk times.  A launch takes as long as its fullest compute
// unit, a compute unit works through its workgroups' chunks one after the other (its two resident workgroups
// share the pipe), and every workgroup adds about six chunk times of prologue and epilogue.  One piece means whole
// tiles with the tail shared out evenly (plan_tail); it stays unless splitting is at least 3 % cheaper, but not
// below 32 tiles, where the fix-up kernel would add up too many slots per tile.  Splits are tried from four
// workgroups per compute unit (enough requests in flight when the layer is bound by memory) up to 4096
// workgroups, with at least four chunks each.
// bf16 (chunks so short that latency is the limit): measured best with about 1024 workgroups, whatever the tiles.
int choose_splits(int64_t tiles, int64_t nch, bool pipe_bound, int min_rounds = 2) {
  const int64_t S = chip_slots(), cus = S / 2;
  const double c0 = 6.0;
  if (tiles < 1) tiles = 1;
  const int64_t cap = nch / 4 > 0 ? nch / 4 : 1;
  // at least min_rounds workgroups per workgroup slot
  const int64_t lo = std::min(cap, (min_rounds * S + tiles - 1) / tiles), hi = std::min(cap, std::max<int64_t>(1, 4096 / tiles));
  if (!pipe_bound) return (int)std::max<int64_t>(1, lo);
  double best = tiles >= 32 ? 0.97 * (double)tiles / (double)cus * ((double)nch + c0) : 1e300;
  int64_t bestS = 1;
  for (int64_t sp = std::max<int64_t>(2, lo); sp <= hi; ++sp) {
    const int64_t rounds = (tiles * sp + cus - 1) / cus, per = (nch + sp - 1) / sp;
    const double c = (double)rounds * ((double)per + c0) + 0.02 * (double)sp;
    if (c < best) { best = c; bestS = sp; }
  }
  return (int)bestS;
}

// Floats of split partials a weight-gradient call on Ks kernels may need, and never fewer than any call on fewer
// kernels of the same layer needs (the split count grows as the slice shrinks).  A call makes one launch for its
// full row tiles and one for a half tile; the launches follow each other and use the same place.
int64_t split_partial_elems(const Geo& g, int CT, int64_t nch, bool pipe_bound, int min_rounds = 2) {
  int64_t need = 0;
  for (int t = 1; t <= (g.Ks + cs::BM - 1) / cs::BM; ++t) {
    const int64_t rows = std::min<int64_t>(g.Ks, (int64_t)t * cs::BM);
    const int sp = choose_splits((int64_t)t * CT, nch, pipe_bound, min_rounds);
    if (sp > 1) need = std::max(need, (int64_t)sp * rows * g.CRS);
  }
  if (pipe_bound && g.Ks > 0) {   // the 64- or 96-row tile for the rest (fp32 kernels only)
    const int sp = choose_splits(CT, nch, pipe_bound, min_rounds);
    if (sp > 1) need = std::max(need, (int64_t)sp * std::min(g.Ks, 96) * g.CRS);
  }
  return need;
}

// Workgroups of a weight-gradient launch: one per (tile, split) when the reduction is split, else the whole tiles
// plus the workgroups that share the tail.
unsigned split_grid(int tiles, int splits, const cs::TailPlan& tail) {
  if (splits > 1) return (unsigned)cs::grid_contiguous(tiles * splits);
  return (unsigned)(cs::grid_contiguous(tail.nFull) + cs::grid_contiguous(tail.nTailWg));
}

struct BwdWeightPlan {
  int MB, CT, nch;
  size_t off_xt, off_dyt, off_part, off_tail, total;
};

BwdWeightPlan plan_bwd_weight(const Geo& g) {
  BwdWeightPlan p;
  p.MB = (g.Ks + cs::BM - 1) / cs::BM;
  p.CT = (g.CRS + cs::BN - 1) / cs::BN;
  p.nch = g.PQ * g.NB;
  size_t o = kZeroBytes;
  p.off_xt = o;   o += seg((int64_t)g.C * g.HW * g.Np);
  p.off_dyt = o;  o += seg((int64_t)g.Ks * g.PQ * g.Np);
  // split partials or tail slots: a launch uses one of them, in the same place
  p.off_part = p.off_tail = o;
  o += std::max(seg(split_partial_elems(g, p.CT, p.nch, true)), tail_bytes(p.nch));
  p.total = o;
  return p;
}

// One-shot timing probe, per host thread (see conv_probe_next_call).
thread_local hipEvent_t tl_probe_start = nullptr;
thread_local hipEvent_t tl_probe_stop = nullptr;

struct Probe {
  hipEvent_t start, stop;
  Probe() : start(tl_probe_start), stop(tl_probe_stop) { tl_probe_start = tl_probe_stop = nullptr; }
  void begin(hipStream_t st) const { if (start && stop) (void)hipEventRecord(start, st); }
  void end(hipStream_t st) const { if (start && stop) (void)hipEventRecord(stop, st); }
};

// ---- bfloat16 matrix-core paths (packed bf16 work copies, see gemm_bf16_kernels.h) ----
inline size_t seg16(int64_t halves) { return (size_t)round_up(halves * 2, 256); }

// Forward pass and input gradient pad the channels to 64 in their channel-innermost copies (forward) or fill C of a
// tile's 128 rows (input gradient).  The instruction is sixteen times as dense as the fp32 one, so that still pays
// down to 8 channels (measured against the fp32 kernels on converted operands: 16 channels 7x7 0.42 -> 0.27 ms per
// step, 8 channels 9x9 0.43 -> 0.32 ms, 17 channels 3x3 0.182 -> 0.173 ms; 4 channels 11x11: forward 0.096 -> 0.127 ms).
// Layers with at most 16 channels come here only when the few-channel path does not take them.
constexpr int kBf16MinChannels = 8;
bool bf16_mfma_fwd_ok(const Geo& g, int dtype) {
  const int64_t Cp = round_up(g.C, 64);
  return dtype == CONV_BF16 && g.C >= kBf16MinChannels && (int64_t)g.HW * g.Np * Cp < kMaxElems &&
         (int64_t)g.Ks * g.RS * Cp < kMaxElems;
}
bool bf16_mfma_bwd_data_ok(const Geo& g, int dtype) {
  const int64_t Ksp = round_up(g.Ks, 64);
  return dtype == CONV_BF16 && g.C >= kBf16MinChannels && (int64_t)g.PQ * g.Np * Ksp < kMaxElems &&
         (int64_t)g.RS * g.C * Ksp < kMaxElems;
}
bool bf16_mfma_bwd_weight_ok(const Geo& g, int dtype) {
  const int64_t Np64 = round_up(g.N, 64);
  return dtype == CONV_BF16 && (int64_t)g.C * g.HW * Np64 < kMaxElems && (int64_t)g.Ks * g.PQ * Np64 < kMaxElems;
}

// Sharing a tail of wide tiles moves 256 KB accumulator images through memory: measured on 183 tiles of 36 chunks
// for 256 slots, sharing (10 chunk times of idle slots filled) took 14 us longer than one workgroup per tile.
constexpr int kWideShareCost = 24;
// Workgroup slots and tail scratch of the wide (256 x 256, 128 KB of LDS) bf16 tiles: one workgroup per compute unit.
inline int wide_slots() { return chip_slots() / 2; }
inline size_t wide_tail_bytes(int nch) {
  return nch >= 16 ? (size_t)wide_slots() * 2 * cs::TAIL2_SLOT_FLOATS * 4 : 0;
}
// A slice of more than 128 kernels needs two 128-row tiles anyway; one 256-row tile then computes the same rows
// with half the staged bytes and three quarters of the LDS reads per MFMA.
inline bool wide_rows(int rows) { return rows > cs::BM; }

struct Fwd16Plan {
  bool wide;
  int Cp, nch, MB, CT;
  cs::TailPlan tail;
  size_t off_x, off_w, off_yt, off_zero, off_tail, total;
};
Fwd16Plan plan_fwd16(const Geo& g) {
  Fwd16Plan p;
  p.Cp = (int)round_up(g.C, 64);
  p.nch = g.RS * (p.Cp / cs::BK16);
  p.wide = wide_rows(g.Ks);
  if (p.wide) {
    p.MB = (g.Ks + cs::BM2 - 1) / cs::BM2;
    p.CT = (g.PQ * g.NB + 7) / 8;
    p.tail = plan_tail(p.MB * p.CT, p.nch, wide_slots(), kWideShareCost);
  } else {
    p.MB = (g.Ks + cs::BM - 1) / cs::BM;
    p.CT = (g.PQ * g.NB + 3) / 4;
    p.tail = plan_tail(p.MB * p.CT, p.nch);
  }
  size_t o = kZeroBytes;
  p.off_x = o;    o += seg16((int64_t)g.HW * g.Np * p.Cp);
  p.off_w = o;    o += seg16((int64_t)g.Ks * g.RS * p.Cp);
  p.off_yt = o;   o += seg((int64_t)g.Ks * g.PQ * g.Np);
  p.off_zero = o; o += seg16((int64_t)32 * p.Cp + 64);   // a column block of zeros: 32 images x Cp channels
  p.off_tail = o; o += p.wide ? wide_tail_bytes(p.nch) : tail_bytes(p.nch);
  p.total = o;
  return p;
}

struct BwdData16Plan {
  bool wide;
  int Ksp, MB, CT;
  cs::RunPlan run;
  size_t off_dy, off_w, off_dxt, off_perm, off_pre, off_scratch, off_zero, off_tail, total;
};
BwdData16Plan plan_bwd_data16(const Geo& g) {
  BwdData16Plan p;
  p.Ksp = (int)round_up(g.Ks, 64);
  // Wide tiles when the channels need two 128-row tiles anyway and the tap tables (36 bytes per tap) fit behind
  // the 128 KB of stages.  With fewer wide tiles than compute units the line of tiles is cut into equal runs, and
  // nearly every workgroup then parks two 256 KB accumulator images for the fix-up kernel: that pays only when a
  // run is long (measured: 235 chunks per run 7 % faster than the narrow tiles, 78 chunks 19 % slower).
  p.wide = wide_rows(g.C) && g.RS <= 512;
  if (p.wide) {
    const int MB2 = (g.C + cs::BM2 - 1) / cs::BM2;
    const int64_t CT2 = ((int64_t)g.HW * g.NB + 7) / 8;
    if (MB2 * CT2 < wide_slots()) {
      // taps that reach a pixel, summed over the pixels: (valid (p,r) pairs) x (valid (q,s) pairs)
      int64_t rows = 0, cols = 0;
      for (int pp = 0; pp < g.P; ++pp)
        for (int r = 0; r < g.R; ++r) rows += (unsigned)(pp * g.sh - g.ph + r) < (unsigned)g.H;
      for (int q = 0; q < g.Q; ++q)
        for (int ss = 0; ss < g.S; ++ss) cols += (unsigned)(q * g.sw - g.pw + ss) < (unsigned)g.W;
      const int64_t line = rows * cols * g.NB / 8 * (p.Ksp / cs::BK16);   // chunks on the line of wide tiles, about
      p.wide = line / std::max(1, wide_slots() / MB2) >= 160;
    }
  }
  const int bpt = p.wide ? 8 : 4;
  p.MB = p.wide ? (g.C + cs::BM2 - 1) / cs::BM2 : (g.C + cs::BM - 1) / cs::BM;
  p.CT = (g.HW * g.NB + bpt - 1) / bpt;
  size_t o = kZeroBytes;
  p.off_dy = o;   o += seg16((int64_t)g.PQ * g.Np * p.Ksp);
  p.off_w = o;    o += seg16((int64_t)g.RS * g.C * p.Ksp);
  p.off_dxt = o;  o += seg((int64_t)g.C * g.HW * g.Np);
  p.off_perm = o; o += seg(g.HW);
  p.off_pre = o;  o += seg((int64_t)(g.HW * g.NB + 3) / 4 + 2);   // room for the narrow tiles' line, whatever the choice
  p.off_scratch = o; o += seg(cs::po::axes_ints(g.H, g.W));
  p.off_zero = o; o += seg16((int64_t)32 * p.Ksp + 64);   // a column block of zeros: 32 images x Ksp kernels
  // With chunks this short the scratch round trip of the cut tiles costs about as much as uneven tiles do, so
  // the runs are used only where one workgroup per tile would leave slots empty.
  const int S = p.wide ? wide_slots() : chip_slots();
  const bool few = (int64_t)p.MB * p.CT < S;
  p.run = plan_runs(p.MB, few && (int64_t)p.CT * g.RS * (p.Ksp / cs::BK16) < (int64_t)1 << 30, S);
  p.off_tail = o;
  o += few ? (size_t)S * 2 * (p.wide ? cs::TAIL2_SLOT_FLOATS : cs::TAIL_SLOT_FLOATS) * 4 : 0;
  p.total = o;
  return p;
}

struct BwdWeight16Plan {
  bool wide;
  int Np64, MB, CT, nch, splits, chPerSplit;
  cs::TailPlan tail;
  size_t off_xt, off_dyt, off_part, off_tail, total;
};
// Tile shape and split count of the bf16 weight gradient on a slice of ks kernels.
struct Split16 {
  bool wide;
  int MB, CT, splits;
};
Split16 split16_for(const Geo& g, int ks, int64_t nch) {
  Split16 s;
  s.wide = wide_rows(ks);
  s.MB = s.wide ? (ks + cs::BM2 - 1) / cs::BM2 : (ks + cs::BM - 1) / cs::BM;
  s.CT = s.wide ? (g.CRS + cs::BN2 - 1) / cs::BN2 : (g.CRS + cs::BN - 1) / cs::BN;
  // about 1024 narrow workgroups (two rounds of two per compute unit) or 512 wide ones (two rounds of one); from a
  // quarter as many wide tiles as compute units on, the reduction is not split but the tiles are shared out in
  // equal runs (measured on 98 tiles: 0.24 ms in six splits, 0.20 ms in two, less in runs)
  const int64_t tiles = (int64_t)s.MB * s.CT;
  s.splits = s.wide ? (tiles >= wide_slots() / 4 ? 1 : choose_splits(tiles, nch, false, 1)) : choose_splits(tiles, nch, false, 2);
  return s;
}
// Floats of split partials such a call may need, and never fewer than a call on fewer kernels of the same layer
// needs (the split count grows as the slice shrinks).
int64_t split_partial_elems16(const Geo& g, int64_t nch) {
  int64_t need = 0;
  for (int ks = 1; ks <= g.Ks; ++ks) {
    const int sp = split16_for(g, ks, nch).splits;
    if (sp > 1) need = std::max(need, (int64_t)sp * ks * g.CRS);
  }
  return need;
}
BwdWeight16Plan plan_bwd_weight16(const Geo& g) {
  BwdWeight16Plan p;
  p.Np64 = (int)round_up(g.N, 64);
  p.nch = g.PQ * (p.Np64 / cs::BK16);
  const Split16 sp = split16_for(g, g.Ks, p.nch);
  p.wide = sp.wide; p.MB = sp.MB; p.CT = sp.CT; p.splits = sp.splits;
  const int64_t tiles = (int64_t)p.MB * p.CT;
  p.chPerSplit = (p.nch + p.splits - 1) / p.splits;
  p.splits = (p.nch + p.chPerSplit - 1) / p.chPerSplit;   // whole blocks of chPerSplit chunks: no empty split
  if (p.splits > 1) {
    p.tail.nFull = (int)tiles; p.tail.nTail = 0; p.tail.units = 1; p.tail.nTailWg = 0;
  } else {
    p.tail = p.wide ? plan_tail((int)tiles, p.nch, wide_slots(), kWideShareCost) : plan_tail((int)tiles, p.nch);
  }
  size_t o = kZeroBytes;
  p.off_xt = o;   o += seg16((int64_t)g.C * g.HW * p.Np64);
  p.off_dyt = o;  o += seg16((int64_t)g.Ks * g.PQ * p.Np64);
  p.off_part = p.off_tail = o;   // split partials or tail slots: a call uses one of them
  o += std::max(seg(split_partial_elems16(g, p.nch)), p.wide ? wide_tail_bytes(p.nch) : tail_bytes(p.nch));
  p.total = o;
  return p;
}

inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

int check_launch() { return hipGetLastError() == hipSuccess ? CONV_OK : CONV_ERR_LAUNCH; }

// Raises a kernel's dynamic-LDS limit (needed above 64 KB).  The attribute is per kernel and
// device, so it is set once per (kernel, device, size) and remembered.
template <typename K>
int allow_big_lds(K kernel, int bytes) {
  struct Done { const void* fn; int dev; int bytes; };
  static Done done[32];
  static int ndone = 0;
  static std::mutex mu;
  const std::lock_guard<std::mutex> lock(mu);
  int dev = 0;
  (void)hipGetDevice(&dev);
  for (int i = 0; i < ndone; ++i)
    if (done[i].fn == (const void*)kernel && done[i].dev == dev && done[i].bytes >= bytes) return CONV_OK;
  if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return CONV_ERR_LAUNCH;
  if (ndone < 32) done[ndone++] = Done{(const void*)kernel, dev, bytes};
  return CONV_OK;
}

// True when some window reaches outside the image, i.e. taps must be range-checked.
bool needs_pad_checks(const Geo& g) {
  return g.ph > 0 || g.pw > 0 || (g.P - 1) * g.sh - g.ph + g.R > g.H || (g.Q - 1) * g.sw - g.pw + g.S > g.W;
}

// ---- pixel-major path for layers with few input channels (pm_kernels.h) ----
// Chosen for the whole layer (never by the slice), so that every slice of a layer takes the same path.
struct PmPlan {
  bool ok;        // forward and weight gradient can take the path
  bool ok_data;   // the input gradient too (its T = w^T * dy matrix fits)
  bool copy;      // taps are read from a zero-bordered fp32 copy of x (padding, or bf16 input) instead of x itself
  cs::PmGeo pg;
};
PmPlan plan_pm(const Geo& g, int dtype) {
  PmPlan p;
  const bool pad = needs_pad_checks(g);
  p.copy = pad || dtype != CONV_F32;
  p.pg.Hp = pad ? (g.P - 1) * g.sh + g.R : g.H;
  p.pg.Wp = pad ? (g.Q - 1) * g.sw + g.S : g.W;
  p.pg.NPQ = (int)std::min<int64_t>((int64_t)g.N * g.PQ, INT32_MAX);
  p.pg.CT = (p.pg.NPQ + cs::BN - 1) / cs::BN;
  p.pg.NC = (g.PQ + 31) / 32;
  p.ok = g.C <= 16 && g.CRS <= 480 && g.PQ >= 32 && (int64_t)g.N * g.C * p.pg.Hp * p.pg.Wp < kMaxElems;
  p.ok_data = p.ok && (int64_t)g.N * g.CRS * g.PQ < kMaxElems;
  return p;
}

struct PmFwdPlan {
  bool repitch;
  int ldw, nch;
  size_t off_xb, off_w, off_tab, total;
};
PmFwdPlan plan_pm_fwd(const Geo& g, const PmPlan& pm, int dtype) {
  PmFwdPlan p;
  p.repitch = dtype != CONV_F32 || (g.CRS % cs::BK) != 0;
  p.ldw = (int)round_up(g.CRS, cs::BK);
  p.nch = p.ldw / cs::BK;
  size_t o = 0;
  p.off_xb = o;  o += pm.copy ? seg((int64_t)g.N * g.C * pm.pg.Hp * pm.pg.Wp) : 0;
  p.off_w = o;   o += p.repitch ? seg((int64_t)g.Ks * p.ldw) : 0;
  p.off_tab = o; o += seg((int64_t)(p.nch + 4) * cs::BK);
  p.total = o;
  return p;
}

// bf16 forward pass of a few-channel layer on the bf16 matrix cores (fwd16_pm_gemm_kernel).
struct Pm16Plan {
  bool ok;
  cs::Pm16Geo pg;
  int nch, MB, CT, NPQ;
  int64_t ldw;
  size_t off_xc, off_wk, total;
};
Pm16Plan plan_pm16_fwd(const Geo& g, const PmPlan& pm, int dtype) {
  Pm16Plan p;
  p.pg.Cp = (g.C <= 4 && g.sw % 2 == 0) ? 4 : g.C <= 8 ? 8 : 16;   // 4: windows must start on 16-byte boundaries
  p.pg.WPC = cs::BK16 / p.pg.Cp;
  p.pg.CPR = (g.S + p.pg.WPC - 1) / p.pg.WPC;
  p.pg.Hb = (g.P - 1) * g.sh + g.R;
  p.pg.Wb = (g.Q - 1) * g.sw + p.pg.CPR * p.pg.WPC;
  p.nch = g.R * p.pg.CPR;
  p.ldw = (int64_t)p.nch * cs::BK16;
  p.NPQ = pm.pg.NPQ;
  p.MB = (g.Ks + cs::BM - 1) / cs::BM;
  p.CT = (p.NPQ + cs::BN - 1) / cs::BN;
  const int64_t xc_elems = (int64_t)g.N * p.pg.Hb * p.pg.Wb * p.pg.Cp;
  p.ok = dtype == CONV_BF16 && pm.ok && g.C <= 16 && xc_elems < kMaxElems && (int64_t)g.Ks * p.ldw < kMaxElems &&
         (int64_t)p.MB * p.CT < ((int64_t)1 << 30);
  size_t o = 0;
  p.off_xc = o; o += seg16(xc_elems);
  p.off_wk = o; o += seg16((int64_t)g.Ks * p.ldw);
  p.total = o;
  return p;
}

// Images per pass over T: T = w^T dy is four bytes per (tap, channel, pixel), many times the size of dy and dx,
// and is written once and read once.  Computed for a group of images at a time, with the sum over taps following
// each group, a T of more than the chip's 256 MB memory-side cache stays in that cache between the two kernels
// instead of going out to memory and back (64 images of 3 x 224 x 224 under 11 x 11 stride 4, T = 281 MB: the bf16
// input gradient takes 0.222 ms in one pass, 0.181 ms in two groups; groups of a quarter of the cache are slower
// than one pass, the launches get too short).
constexpr int64_t kPmTGroupBytes = (int64_t)160 << 20;
int pm_T_group(const Geo& g) {
  const int64_t bytes = (int64_t)g.N * g.CRS * g.PQ * 4;
  const int64_t groups = (bytes + kPmTGroupBytes - 1) / kPmTGroupBytes;
  return (int)((g.N + groups - 1) / groups);
}

struct PmBwdDataPlan {
  bool mfma16;   // bf16: T on the bf16 matrix cores from a channels-last copy of the slice's maps
  int Ksp, nch;
  size_t off_dy, off_wt, off_T, total;
};
PmBwdDataPlan plan_pm_bwd_data(const Geo& g, int dtype) {
  PmBwdDataPlan p;
  const int64_t Kp16 = round_up(g.Ks, cs::BK16);
  p.mfma16 = dtype == CONV_BF16 && (int64_t)g.N * g.PQ * Kp16 < kMaxElems && (int64_t)g.CRS * Kp16 < kMaxElems;
  size_t o = 0;
  if (p.mfma16) {
    p.Ksp = (int)Kp16;
    p.nch = p.Ksp / cs::BK16;
    p.off_dy = o; o += seg16((int64_t)g.N * g.PQ * p.Ksp);
    p.off_wt = o; o += seg16((int64_t)g.CRS * p.Ksp);
    p.off_T = o;  o += seg((int64_t)pm_T_group(g) * g.CRS * g.PQ);   // one group of images at a time
    p.total = o;
    return p;
  }
  p.Ksp = (int)round_up(g.Ks, cs::BK);
  p.nch = p.Ksp / cs::BK;
  p.off_dy = o; o += dtype != CONV_F32 ? seg((int64_t)g.N * g.Ks * g.PQ) : 0;   // fp32 copy of the slice's maps
  p.off_wt = o; o += seg((int64_t)g.CRS * p.Ksp);
  p.off_T = o;  o += seg((int64_t)pm_T_group(g) * g.CRS * g.PQ);   // one group of images at a time
  p.total = o;
  return p;
}

// Workgroups per workgroup slot the pixel-major weight gradient is split into at least (its operands sit in
// the caches, so one round of long pieces beats several rounds of short ones).
constexpr int kPmSplitRounds = 1;
struct PmBwdWeightPlan {
  int CT, nch;
  size_t off_xb, off_pix, off_part, total;
};
PmBwdWeightPlan plan_pm_bwd_weight(const Geo& g, const PmPlan& pm) {
  PmBwdWeightPlan p;
  p.CT = (g.CRS + cs::BN - 1) / cs::BN;
  p.nch = g.N * pm.pg.NC;
  size_t o = kZeroBytes;
  p.off_xb = o;   o += pm.copy ? seg((int64_t)g.N * g.C * pm.pg.Hp * pm.pg.Wp) : 0;
  p.off_pix = o;  o += seg((int64_t)pm.pg.NC * 32);
  p.off_part = o; o += seg(split_partial_elems(g, p.CT, p.nch, true, kPmSplitRounds));
  p.total = o;
  return p;
}

// src[rows][cols] (pitch srcPitch, element type by dtype) -> dst[cols][rowsPad] (fp32, or bf16 when
// out16), for batches 0..batch-1; batches at or past batchValid are written as zeros.
void launch_transpose_in(int dtype, const void* src, int64_t srcBatch, int64_t srcPitch, int rows, int cols,
                         void* dst, int64_t dstBatch, int64_t dstPitch, int rowsPad, int batch,
                         float* zero_page, hipStream_t st, bool out16 = false, int batchValid = -1, int group = 0,
                         int interleave = 0) {
  if (batchValid < 0) batchValid = batch;
  for (int b0 = 0; b0 < batch; b0 += 32768) {  // grid.z is limited to 65535
    const int nb = batch - b0 < 32768 ? batch - b0 : 32768;
    const dim3 grid((cols + 63) / 64, (rowsPad + 63) / 64, nb);
    float* zp = b0 == 0 ? zero_page : nullptr;
    const size_t ain = dtype == CONV_F32 ? 16 : 8, aout = out16 ? 8 : 16;   // four elements
    const bool vec4 = (uintptr_t)src % ain == 0 && (uintptr_t)dst % aout == 0 && cols % 4 == 0 && rowsPad % 4 == 0 &&
                      (srcPitch | srcBatch | dstPitch | dstBatch) % 4 == 0;
#define CS_LAUNCH_TRANSPOSE_IN(KERNEL, TIN, TOUT)                                                                  \
  hipLaunchKernelGGL((KERNEL<TIN, TOUT>), grid, dim3(256), 0, st, (const TIN*)src, srcBatch, srcPitch, rows, cols, \
                     (TOUT*)dst, dstBatch, dstPitch, rowsPad, b0, batchValid, zp, group, interleave)
    if (dtype == CONV_F32 && !out16) {
      if (vec4) CS_LAUNCH_TRANSPOSE_IN(cs::transpose_in_v4_kernel, float, float);
      else CS_LAUNCH_TRANSPOSE_IN(cs::transpose_in_kernel, float, float);
    } else if (dtype == CONV_F32) {
      if (vec4) CS_LAUNCH_TRANSPOSE_IN(cs::transpose_in_v4_kernel, float, uint16_t);
      else CS_LAUNCH_TRANSPOSE_IN(cs::transpose_in_kernel, float, uint16_t);
    } else if (!out16) {
      if (vec4) CS_LAUNCH_TRANSPOSE_IN(cs::transpose_in_v4_kernel, uint16_t, float);
      else CS_LAUNCH_TRANSPOSE_IN(cs::transpose_in_kernel, uint16_t, float);
    } else {
      if (vec4) CS_LAUNCH_TRANSPOSE_IN(cs::transpose_in_v4_kernel, uint16_t, uint16_t);
      else CS_LAUNCH_TRANSPOSE_IN(cs::transpose_in_kernel, uint16_t, uint16_t);
    }
#undef CS_LAUNCH_TRANSPOSE_IN
  }
}

// src[cols][srcPitch] fp32 -> dst[rows][cols] (pitch dstPitch), optionally accumulating.
void launch_transpose_out(int dtype, bool acc, const float* src, int64_t srcPitch, int rows, int cols,
                          void* dst, int64_t dstPitch, hipStream_t st) {
  const dim3 grid((cols + 63) / 64, (rows + 63) / 64);
  const size_t aout = dtype == CONV_F32 ? 16 : 8;   // four elements
  const bool vec4 = (uintptr_t)src % 16 == 0 && (uintptr_t)dst % aout == 0 && cols % 4 == 0 &&
                    (srcPitch | dstPitch) % 4 == 0;
#define CS_LAUNCH_TRANSPOSE_OUT(KERNEL, TOUT, ACC) \
  hipLaunchKernelGGL((KERNEL<TOUT, ACC>), grid, dim3(256), 0, st, src, srcPitch, rows, cols, (TOUT*)dst, dstPitch)
  if (dtype == CONV_F32) {
    if (vec4 && acc) CS_LAUNCH_TRANSPOSE_OUT(cs::transpose_out_v4_kernel, float, true);
    else if (vec4) CS_LAUNCH_TRANSPOSE_OUT(cs::transpose_out_v4_kernel, float, false);
    else if (acc) CS_LAUNCH_TRANSPOSE_OUT(cs::transpose_out_kernel, float, true);
    else CS_LAUNCH_TRANSPOSE_OUT(cs::transpose_out_kernel, float, false);
  } else {
    if (vec4 && acc) CS_LAUNCH_TRANSPOSE_OUT(cs::transpose_out_v4_kernel, uint16_t, true);
    else if (vec4) CS_LAUNCH_TRANSPOSE_OUT(cs::transpose_out_v4_kernel, uint16_t, false);
    else if (acc) CS_LAUNCH_TRANSPOSE_OUT(cs::transpose_out_kernel, uint16_t, true);
    else CS_LAUNCH_TRANSPOSE_OUT(cs::transpose_out_kernel, uint16_t, false);
  }
#undef CS_LAUNCH_TRANSPOSE_OUT
}

inline size_t elem_size(int dtype) { return dtype == CONV_F32 ? 4 : 2; }

int check_ws(const void* ws, size_t ws_bytes, size_t need) {
  if (need == 0) return CONV_OK;
  if (!ws || ws_bytes < need || misaligned(ws, 256)) return CONV_ERR_WORKSPACE;
  return CONV_OK;
}

// ---- pixel-major passes: host side ----
inline int grid_for(int64_t count, int cap = 8192) { return (int)std::min<int64_t>((count + 255) / 256, cap); }
// Persistent workgroups for a stream kernel over `tiles` tiles: one per workgroup slot, fewer when there are fewer tiles.
inline unsigned stream_grid(int64_t tiles) { return (unsigned)cs::grid_contiguous((int)std::min<int64_t>(tiles, chip_slots())); }

// The image the taps are read from: x itself, or its zero-bordered fp32 copy (made here).
const float* pm_input(const Geo& g, const PmPlan& pm, int dtype, const void* x, float* xb, hipStream_t st,
                      bool ready = false) {
  if (!pm.copy) return (const float*)x;
  if (ready) return xb;
  const int64_t count = (int64_t)g.N * g.C * pm.pg.Hp * pm.pg.Wp;
  if (dtype == CONV_F32)
    hipLaunchKernelGGL(cs::pm_border_copy_kernel<float>, dim3(grid_for(count)), dim3(256), 0, st, g, pm.pg.Hp, pm.pg.Wp,
                       (const float*)x, xb);
  else
    hipLaunchKernelGGL(cs::pm_border_copy_kernel<uint16_t>, dim3(grid_for(count)), dim3(256), 0, st, g, pm.pg.Hp,
                       pm.pg.Wp, (const uint16_t*)x, xb);
  return xb;
}

int pm16_fwd(const Geo& g, const Pm16Plan& p, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
             hipStream_t st, const Probe& probe, bool input_ready) {
  int rc;
  if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
  char* base = (char*)ws;
  uint16_t* xc = (uint16_t*)(base + p.off_xc);
  uint16_t* wk = (uint16_t*)(base + p.off_wk);
  if (!input_ready) {
    const int blocks = grid_for((int64_t)g.N * p.pg.Hb * p.pg.Wb, 1 << 20);
    if (p.pg.Cp == 4)
      hipLaunchKernelGGL(cs::pm16_channels_last_kernel<4>, dim3(blocks), dim3(256), 0, st, g, p.pg, (const uint16_t*)x, xc);
    else if (p.pg.Cp == 8)
      hipLaunchKernelGGL(cs::pm16_channels_last_kernel<8>, dim3(blocks), dim3(256), 0, st, g, p.pg, (const uint16_t*)x, xc);
    else
      hipLaunchKernelGGL(cs::pm16_channels_last_kernel<16>, dim3(blocks), dim3(256), 0, st, g, p.pg, (const uint16_t*)x, xc);
  }
  hipLaunchKernelGGL(cs::pm16_filters_kernel, dim3(grid_for((int64_t)g.Ks * p.ldw)), dim3(256), 0, st, g, p.pg,
                     (const uint16_t*)w + (size_t)g.k0 * g.CRS, wk);
  if ((rc = allow_big_lds(cs::fwd16_pm_gemm_kernel, cs::SMEM_BYTES)) != CONV_OK) return rc;
  probe.begin(st);
  hipLaunchKernelGGL(cs::fwd16_pm_gemm_kernel, dim3(cs::grid_contiguous(p.MB * p.CT)), dim3(cs::NT), cs::SMEM_BYTES, st, g,
                     p.pg, wk, p.ldw, xc, (uint16_t*)y, p.NPQ, p.MB, p.CT, p.nch);
  probe.end(st);
  return check_launch();
}

int pm_fwd(const Geo& g, const PmPlan& pm, int dtype, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
           hipStream_t st, const Probe& probe, bool input_ready) {
  const PmFwdPlan p = plan_pm_fwd(g, pm, dtype);
  int rc;
  if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
  char* base = (char*)ws;
  const size_t es = elem_size(dtype);
  const float* xb = pm_input(g, pm, dtype, x, (float*)(base + p.off_xb), st, input_ready);
  const float* wmat;
  int* tab = (int*)(base + p.off_tab);
  const int entries = (p.nch + 4) * cs::BK;
  const int tblocks = (entries + 255) / 256;
  if (p.repitch) {   // filter rows to fp32 rows of pitch ldw and the tap table, one launch
    float* wp = (float*)(base + p.off_w);
    const char* wsrc = (const char*)w + (size_t)g.k0 * g.CRS * es;
    const int rblocks = grid_for((int64_t)g.Ks * p.ldw, 4096);
    if (dtype == CONV_F32)
      hipLaunchKernelGGL(cs::pm_fwd_setup_kernel<float>, dim3(rblocks + tblocks), dim3(256), 0, st, g, (const float*)wsrc,
                         wp, p.ldw, rblocks, pm.pg.Hp, pm.pg.Wp, entries, tab);
    else
      hipLaunchKernelGGL(cs::pm_fwd_setup_kernel<uint16_t>, dim3(rblocks + tblocks), dim3(256), 0, st, g,
                         (const uint16_t*)wsrc, wp, p.ldw, rblocks, pm.pg.Hp, pm.pg.Wp, entries, tab);
    wmat = wp;
  } else {
    wmat = (const float*)w + (size_t)g.k0 * g.CRS;
    hipLaunchKernelGGL(cs::pm_tap_table_kernel, dim3(tblocks), dim3(256), 0, st, g, pm.pg.Hp, pm.pg.Wp, entries, tab);
  }
  const RowSplit rs = split_rows(g.Ks, true);
  probe.begin(st);
  auto launch = [&](auto kern, auto* yout, int m0, int tiles) -> int {
    int rc2;
    if ((rc2 = allow_big_lds(kern, cs::SMEM_BYTES)) != CONV_OK) return rc2;
    hipLaunchKernelGGL(kern, dim3(stream_grid((int64_t)tiles * pm.pg.CT)), dim3(cs::NT), cs::SMEM_BYTES, st, g, pm.pg,
                       wmat, p.ldw, xb, tab, yout, m0, tiles, p.nch);
    return CONV_OK;
  };
  rc = CONV_OK;
  if (dtype == CONV_F32) {
    if (rs.full > 0) rc = launch(cs::fwd_pm_gemm_kernel<2, float>, (float*)y, 0, rs.full);
    if (rc == CONV_OK && rs.last == 1) rc = launch(cs::fwd_pm_gemm_kernel<1, float>, (float*)y, rs.full * cs::BM, 1);
    if (rc == CONV_OK && rs.last == 3) rc = launch(cs::fwd_pm_gemm_kernel<3, float>, (float*)y, rs.full * cs::BM, rs.nlast);
  } else {
    if (rs.full > 0) rc = launch(cs::fwd_pm_gemm_kernel<2, uint16_t>, (uint16_t*)y, 0, rs.full);
    if (rc == CONV_OK && rs.last == 1) rc = launch(cs::fwd_pm_gemm_kernel<1, uint16_t>, (uint16_t*)y, rs.full * cs::BM, 1);
    if (rc == CONV_OK && rs.last == 3) rc = launch(cs::fwd_pm_gemm_kernel<3, uint16_t>, (uint16_t*)y, rs.full * cs::BM, rs.nlast);
  }
  probe.end(st);
  if (rc != CONV_OK) return rc;
  return check_launch();
}

int pm_bwd_data(const Geo& gAll, const PmPlan& pmAll, int dtype, bool acc, const void* dy, const void* w, void* dx, void* ws,
                size_t ws_bytes, hipStream_t st, const Probe& probe) {
  const PmBwdDataPlan p = plan_pm_bwd_data(gAll, dtype);
  int rc;
  if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
  char* base = (char*)ws;
  const size_t es = elem_size(dtype);
  float* T = (float*)(base + p.off_T);
  const int NG = pm_T_group(gAll);
  // operands that do not depend on the group
  uint16_t* dyc = (uint16_t*)(base + p.off_dy);
  uint16_t* wt16 = (uint16_t*)(base + p.off_wt);
  float* wt = (float*)(base + p.off_wt);
  const float* dy_k0 = nullptr;
  int64_t imgPitch = 0;
  if (p.mfma16) {
    // dy[n][k0+k][pix] -> dyc[n][pix][Ksp] and w[k0+k][(c,r,s)] -> wt[(c,r,s)][Ksp], both bf16, zero past Ks
    launch_transpose_in(dtype, (const uint16_t*)dy + (size_t)gAll.k0 * gAll.PQ, (int64_t)gAll.K * gAll.PQ, gAll.PQ, gAll.Ks,
                        gAll.PQ, dyc, (int64_t)gAll.PQ * p.Ksp, p.Ksp, p.Ksp, gAll.N, nullptr, st, true);
    launch_transpose_in(dtype, (const uint16_t*)w + (size_t)gAll.k0 * gAll.CRS, 0, gAll.CRS, gAll.Ks, gAll.CRS, wt16, 0,
                        p.Ksp, p.Ksp, 1, nullptr, st, true);
    if ((rc = allow_big_lds(cs::bwd_data16_pm_gemm_kernel, cs::SMEM_BYTES)) != CONV_OK) return rc;
  } else {
    // the slice's maps in fp32: dy in place, or a compact copy of the slice's channels for bf16
    if (dtype == CONV_F32) {
      dy_k0 = (const float*)dy + (size_t)gAll.k0 * gAll.PQ;
      imgPitch = (int64_t)gAll.K * gAll.PQ;
    } else {
      float* d = (float*)(base + p.off_dy);
      imgPitch = (int64_t)gAll.Ks * gAll.PQ;
      hipLaunchKernelGGL(cs::pm_slice_to_f32_kernel, dim3(grid_for((int64_t)gAll.N * imgPitch)), dim3(256), 0, st,
                         (const uint16_t*)dy + (size_t)gAll.k0 * gAll.PQ, (int64_t)gAll.K * gAll.PQ, imgPitch, gAll.N, d);
      dy_k0 = d;
    }
    // w[k][(c,r,s)] -> wt[(c,r,s)][Ksp], zero past Ks
    launch_transpose_in(dtype, (const char*)w + (size_t)gAll.k0 * gAll.CRS * es, 0, gAll.CRS, gAll.Ks, gAll.CRS, wt, 0, p.Ksp,
                        p.Ksp, 1, nullptr, st);
  }
  for (int n0 = 0; n0 < gAll.N; n0 += NG) {
    // the probe brackets the matrix-core kernels of all groups (and so the sums over taps between them)
    if (n0 == 0) probe.begin(st);
    const bool last_group = n0 + NG >= gAll.N;
    Geo g = gAll;
    g.N = std::min(NG, gAll.N - n0);
    PmPlan pm = pmAll;
    pm.pg.NPQ = g.N * g.PQ;
    pm.pg.CT = (pm.pg.NPQ + cs::BN - 1) / cs::BN;
    if (p.mfma16) {
      const int MB = (g.CRS + cs::BM - 1) / cs::BM;
      hipLaunchKernelGGL(cs::bwd_data16_pm_gemm_kernel, dim3(cs::grid_contiguous(MB * pm.pg.CT)), dim3(cs::NT), cs::SMEM_BYTES,
                         st, wt16, p.Ksp, g.CRS, dyc + (size_t)n0 * g.PQ * p.Ksp, T, g.PQ, pm.pg.NPQ, MB, pm.pg.CT);
      if (last_group) probe.end(st);
    } else {
      const bool vec4 = g.PQ % 4 == 0;
      const RowSplit rs = split_rows(g.CRS, true);
      const float* dyg = dy_k0 + (size_t)n0 * imgPitch;
      auto launch = [&](auto kern, int m0, int tiles) -> int {
        int rc2;
        if ((rc2 = allow_big_lds(kern, cs::SMEM_BYTES)) != CONV_OK) return rc2;
        hipLaunchKernelGGL(kern, dim3(stream_grid((int64_t)tiles * pm.pg.CT)), dim3(cs::NT), cs::SMEM_BYTES, st, g, pm.pg, wt,
                           p.Ksp, dyg, imgPitch, T, m0, tiles, p.nch);
        return CONV_OK;
      };
      rc = CONV_OK;
      if (vec4) {
        if (rs.full > 0) rc = launch(cs::bwd_data_pm_gemm_kernel<2, true>, 0, rs.full);
        if (rc == CONV_OK && rs.last == 1) rc = launch(cs::bwd_data_pm_gemm_kernel<1, true>, rs.full * cs::BM, 1);
        if (rc == CONV_OK && rs.last == 3) rc = launch(cs::bwd_data_pm_gemm_kernel<3, true>, rs.full * cs::BM, rs.nlast);
      } else {
        if (rs.full > 0) rc = launch(cs::bwd_data_pm_gemm_kernel<2, false>, 0, rs.full);
        if (rc == CONV_OK && rs.last == 1) rc = launch(cs::bwd_data_pm_gemm_kernel<1, false>, rs.full * cs::BM, 1);
        if (rc == CONV_OK && rs.last == 3) rc = launch(cs::bwd_data_pm_gemm_kernel<3, false>, rs.full * cs::BM, rs.nlast);
      }
      if (last_group) probe.end(st);
      if (rc != CONV_OK) return rc;
    }
    // one thread per group of `stride` columns for strides up to 4, else per column
    auto col2im = [&](auto* out0, auto acc_tag) {
      using TO = std::remove_pointer_t<decltype(out0)>;
      constexpr bool A = decltype(acc_tag)::value;
      TO* out = out0 + (size_t)n0 * g.C * g.HW;
      const int nv = g.sw <= 4 ? g.sw : 1;
      const int blocks = (grid_for((int64_t)g.N * g.C * g.H * ((g.W + nv - 1) / nv), 1 << 20) + 7) / 8 * 8;
      // strides 2..4 with at most three taps per axis on any element: the variant with all loads in flight
      const bool few = g.sw >= 2 && g.sw <= 4 && (g.R + g.sh - 1) / g.sh <= 3 && (g.S + g.sw - 1) / g.sw <= 3;
      switch (g.sw <= 4 ? g.sw : 0) {
        case 1: hipLaunchKernelGGL((cs::col2im_pm_kernel<TO, A, 1, false>), dim3(blocks), dim3(256), 0, st, g, T, out); break;
        case 2:
          if (few) hipLaunchKernelGGL((cs::col2im_pm_kernel<TO, A, 2, true>), dim3(blocks), dim3(256), 0, st, g, T, out);
          else hipLaunchKernelGGL((cs::col2im_pm_kernel<TO, A, 2, false>), dim3(blocks), dim3(256), 0, st, g, T, out);
          break;
        case 3:
          if (few) hipLaunchKernelGGL((cs::col2im_pm_kernel<TO, A, 3, true>), dim3(blocks), dim3(256), 0, st, g, T, out);
          else hipLaunchKernelGGL((cs::col2im_pm_kernel<TO, A, 3, false>), dim3(blocks), dim3(256), 0, st, g, T, out);
          break;
        case 4:
          if (few) hipLaunchKernelGGL((cs::col2im_pm_kernel<TO, A, 4, true>), dim3(blocks), dim3(256), 0, st, g, T, out);
          else hipLaunchKernelGGL((cs::col2im_pm_kernel<TO, A, 4, false>), dim3(blocks), dim3(256), 0, st, g, T, out);
          break;
        default: hipLaunchKernelGGL((cs::col2im_pm_kernel<TO, A, 0, false>), dim3(blocks), dim3(256), 0, st, g, T, out); break;
      }
    };
    if (dtype == CONV_F32) {
      if (acc) col2im((float*)dx, std::true_type{});
      else col2im((float*)dx, std::false_type{});
    } else {
      if (acc) col2im((uint16_t*)dx, std::true_type{});
      else col2im((uint16_t*)dx, std::false_type{});
    }
  }
  return check_launch();
}

// fp32 only (bf16 layers take the bf16 matrix-core weight gradient).
int pm_bwd_weight(const Geo& g, const PmPlan& pm, const void* x, const void* dy, void* dw, void* ws, size_t ws_bytes,
                  hipStream_t st, const Probe& probe, bool input_ready) {
  const PmBwdWeightPlan p = plan_pm_bwd_weight(g, pm);
  int rc;
  if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
  char* base = (char*)ws;
  float* zero = (float*)base;
  const float* xb = pm_input(g, pm, CONV_F32, x, (float*)(base + p.off_xb), st, input_ready);
  int* pixtab = (int*)(base + p.off_pix);
  hipLaunchKernelGGL(cs::pm_pixel_table_kernel, dim3((pm.pg.NC * 32 + 255) / 256), dim3(256), 0, st, g, pm.pg.Wp, pm.pg.NC,
                     pixtab, zero);   // clears the zero page too
  const float* dy_k0 = (const float*)dy + (size_t)g.k0 * g.PQ;
  const int64_t imgPitch = (int64_t)g.K * g.PQ;
  float* dwslice = (float*)dw + (size_t)g.k0 * g.CRS;
  float* scratch = (float*)(base + p.off_part);
  auto launch = [&](auto kern, int mi, int m0, int tiles) -> int {
    int rc2;
    if ((rc2 = allow_big_lds(kern, cs::SMEM_BYTES)) != CONV_OK) return rc2;
    const int rows = std::min(g.Ks - m0, tiles * (mi == 3 ? 96 : mi == 4 ? 128 : 64 * mi));
    const int splits = choose_splits((int64_t)tiles * p.CT, p.nch, true, kPmSplitRounds);
    const int64_t stride = (int64_t)rows * g.CRS;
    float* out = splits > 1 ? scratch : dwslice;
    const int rowBase = splits > 1 ? m0 : 0;
    hipLaunchKernelGGL(kern, dim3(cs::grid_contiguous(tiles * p.CT * splits)), dim3(cs::NT), cs::SMEM_BYTES, st, g, pm.pg,
                       dy_k0, imgPitch, xb, zero, pixtab, out, stride, m0, rowBase, tiles, p.CT, p.nch, splits);
    if (splits > 1)
      hipLaunchKernelGGL(cs::splitk_reduce_kernel, dim3(grid_for(stride)), dim3(256), 0, st, scratch, stride, splits,
                         dwslice + (int64_t)m0 * g.CRS, stride);
    return CONV_OK;
  };
  const bool vec4 = g.PQ % 4 == 0;
  const RowSplit rs = split_rows(g.Ks, true);
  rc = CONV_OK;
  const bool narrow = g.CRS <= 96;   // 128 x 96 tiles: a fourth column block would multiply padding
  probe.begin(st);
  if (vec4) {
    if (rs.full > 0) rc = narrow ? launch(cs::bwd_weight_pm_gemm_kernel<4, true>, 4, 0, rs.full)
                                 : launch(cs::bwd_weight_pm_gemm_kernel<2, true>, 2, 0, rs.full);
    if (rc == CONV_OK && rs.last == 1) rc = launch(cs::bwd_weight_pm_gemm_kernel<1, true>, 1, rs.full * cs::BM, 1);
    if (rc == CONV_OK && rs.last == 3) rc = launch(cs::bwd_weight_pm_gemm_kernel<3, true>, 3, rs.full * cs::BM, rs.nlast);
  } else {
    if (rs.full > 0) rc = narrow ? launch(cs::bwd_weight_pm_gemm_kernel<4, false>, 4, 0, rs.full)
                                 : launch(cs::bwd_weight_pm_gemm_kernel<2, false>, 2, 0, rs.full);
    if (rc == CONV_OK && rs.last == 1) rc = launch(cs::bwd_weight_pm_gemm_kernel<1, false>, 1, rs.full * cs::BM, 1);
    if (rc == CONV_OK && rs.last == 3) rc = launch(cs::bwd_weight_pm_gemm_kernel<3, false>, 3, rs.full * cs::BM, rs.nlast);
  }
  probe.end(st);
  if (rc != CONV_OK) return rc;
  return check_launch();
}

}  // namespace

extern "C" {

int conv_output_dims(const conv_desc_t* desc, int32_t* P, int32_t* Q) {
  if (!desc || !P || !Q) return CONV_ERR_NULL;
  Geo g;
  const int rc = make_geo(desc, g);
  if (rc != CONV_OK) return rc;
  *P = g.P;
  *Q = g.Q;
  return CONV_OK;
}

size_t conv_workspace_bytes(const conv_desc_t* desc, int pass) {
  Geo g;
  if (make_geo(desc, g) != CONV_OK) return 0;
  if (g.Ks == 0) return 0;
  const PmPlan pm = plan_pm(g, desc->dtype);
  switch (pass) {
    case CONV_PASS_FWD:
      if (pm.ok) {
        const Pm16Plan p16 = plan_pm16_fwd(g, pm, desc->dtype);
        return p16.ok ? p16.total : plan_pm_fwd(g, pm, desc->dtype).total;
      }
      return bf16_mfma_fwd_ok(g, desc->dtype) ? plan_fwd16(g).total : plan_fwd(g, desc->dtype).total;
    case CONV_PASS_BWD_DATA:
      if (pm.ok_data) return plan_pm_bwd_data(g, desc->dtype).total;
      return bf16_mfma_bwd_data_ok(g, desc->dtype) ? plan_bwd_data16(g).total : plan_bwd_data(g).total;
    case CONV_PASS_BWD_WEIGHT:
      if (bf16_mfma_bwd_weight_ok(g, desc->dtype)) return plan_bwd_weight16(g).total;
      if (pm.ok) return plan_pm_bwd_weight(g, pm).total;
      return plan_bwd_weight(g).total;
    default: return 0;
  }
}

// The forward kernel over all rows of g (g.Ks of them): full row tiles first, then the 64- or 96-row tile for the
// rest, each with its own tail plan; the two launches share the scratch slots (stream order keeps them apart).
int launch_fwd_gemm(const Geo& g, bool pad, const float* wmat, int ldw, const float* xt, const int* tab, int entries,
                    float* out, int CT, int nch, float* partial, hipStream_t st) {
  int rc;
  const RowSplit rs = split_rows(g.Ks, true);
  // one launch over `tiles` row tiles of shape mi from row m0
  auto launch = [&](auto kern, auto fixup, int mi, int m0, int tiles) -> int {
    const int r = allow_big_lds(kern, cs::SMEM_BYTES);
    if (r != CONV_OK) return r;
    const cs::TailPlan tp = plan_tail(tiles * CT, nch);
    hipLaunchKernelGGL(kern, dim3(cs::grid_contiguous(tp.nFull) + cs::grid_contiguous(tp.nTailWg)), dim3(cs::NT),
                       cs::SMEM_BYTES, st, g, wmat, ldw, xt, tab, entries, out, m0, tiles, CT, nch, tp, partial);
    if (tp.nTail > 0)
      hipLaunchKernelGGL(fixup, dim3(tp.nTail, mi == 2 ? 4 : mi == 1 ? 2 : 3), dim3(cs::NT), 0, st, g, partial, out, m0,
                         tiles, CT, nch, tp);
    return CONV_OK;
  };
  const int m1 = rs.full * cs::BM;
  if (rs.full > 0 &&
      (rc = pad ? launch(cs::fwd_gemm_kernel<true, 2>, cs::fwd_tail_fixup_kernel<2>, 2, 0, rs.full)
                : launch(cs::fwd_gemm_kernel<false, 2>, cs::fwd_tail_fixup_kernel<2>, 2, 0, rs.full)) != CONV_OK)
    return rc;
  if (rs.last == 1 &&
      (rc = pad ? launch(cs::fwd_gemm_kernel<true, 1>, cs::fwd_tail_fixup_kernel<1>, 1, m1, 1)
                : launch(cs::fwd_gemm_kernel<false, 1>, cs::fwd_tail_fixup_kernel<1>, 1, m1, 1)) != CONV_OK)
    return rc;
  if (rs.last == 3 &&
      (rc = pad ? launch(cs::fwd_gemm_kernel<true, 3>, cs::fwd_tail_fixup_kernel<3>, 3, m1, rs.nlast)
                : launch(cs::fwd_gemm_kernel<false, 3>, cs::fwd_tail_fixup_kernel<3>, 3, m1, rs.nlast)) != CONV_OK)
    return rc;
  return CONV_OK;
}

}  // extern "C"

namespace {

int fwd_impl(const conv_desc_t* desc, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
             void* hip_stream, bool input_ready) {
  const Probe probe;
  Geo g;
  int rc = make_geo(desc, g);
  if (rc != CONV_OK) return rc;
  if (!x || !w || !y) return CONV_ERR_NULL;
  if (misaligned(x, 16) || misaligned(w, 16) || misaligned(y, 16)) return CONV_ERR_ALIGN;
  if (g.Ks == 0) return CONV_OK;
  const PmPlan pm = plan_pm(g, desc->dtype);
  if (pm.ok) {
    const Pm16Plan p16 = plan_pm16_fwd(g, pm, desc->dtype);
    if (p16.ok) return pm16_fwd(g, p16, x, w, y, ws, ws_bytes, (hipStream_t)hip_stream, probe, input_ready);
    return pm_fwd(g, pm, desc->dtype, x, w, y, ws, ws_bytes, (hipStream_t)hip_stream, probe, input_ready);
  }
  if (bf16_mfma_fwd_ok(g, desc->dtype)) {
    const Fwd16Plan p = plan_fwd16(g);
    if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    char* base = (char*)ws;
    cs::bf16_t* xp = (cs::bf16_t*)(base + p.off_x);
    cs::bf16_t* wp = (cs::bf16_t*)(base + p.off_w);
    float* yt = (float*)(base + p.off_yt);
    float* partial = (float*)(base + p.off_tail);
    // per image: x[n] as a C x HW matrix -> x_hwnc[hw][n][Cp]; images N..Np-1 are zero
    if (!input_ready)
      launch_transpose_in(CONV_BF16, x, (int64_t)g.C * g.HW, g.HW, g.C, g.HW, xp, p.Cp, (int64_t)g.Np * p.Cp, p.Cp,
                          g.Np, (float*)(base + p.off_x - kZeroBytes), st, true, g.N);
    // w[k][c][rs] -> w_krsc[k][rs][Cp]
    hipLaunchKernelGGL(cs::filters_to_krsc_kernel, dim3((p.Cp + 63) / 64, g.Ks), dim3(256), 0, st,
                       (const uint16_t*)w + (size_t)g.k0 * g.CRS, g.C, g.RS, p.Cp, (uint16_t*)wp);
    cs::bf16_t* zero = (cs::bf16_t*)(base + p.off_zero);
    hipLaunchKernelGGL(cs::fill_zero_kernel<uint16_t>, dim3(16), dim3(256), 0, st, zero, (int64_t)32 * p.Cp + 64);
    const dim3 grid(cs::grid_contiguous(p.tail.nFull) + cs::grid_contiguous(p.tail.nTailWg));
    if (p.wide) {
      if ((rc = allow_big_lds(cs::fwd16_wide_gemm_kernel, cs::SMEM2_BYTES)) != CONV_OK) return rc;
      probe.begin(st);
      hipLaunchKernelGGL(cs::fwd16_wide_gemm_kernel, grid, dim3(cs::NT2), cs::SMEM2_BYTES, st, g, wp, p.Cp, xp, zero, yt,
                         p.MB, p.CT, p.nch, p.tail, partial);
      if (p.tail.nTail > 0)
        hipLaunchKernelGGL(cs::fwd16_wide_fixup_kernel, dim3(p.tail.nTail, 8), dim3(cs::NT2), 0, st, g, partial, yt, p.MB,
                           p.CT, p.nch, p.tail);
    } else {
      if ((rc = allow_big_lds(cs::fwd16_gemm_kernel, cs::SMEM_BYTES)) != CONV_OK) return rc;
      probe.begin(st);
      hipLaunchKernelGGL(cs::fwd16_gemm_kernel, grid, dim3(cs::NT), cs::SMEM_BYTES, st, g, wp, p.Cp, xp, zero, yt, p.MB,
                         p.CT, p.nch, p.tail, partial);
      if (p.tail.nTail > 0)
        hipLaunchKernelGGL(cs::fwd_tail_fixup_kernel<2>, dim3(p.tail.nTail, 4), dim3(cs::NT), 0, st, g, partial, yt, 0,
                           p.MB, p.CT, p.nch, p.tail);
    }
    probe.end(st);
    launch_transpose_out(CONV_BF16, false, yt, g.Np, g.N, g.Ks * g.PQ, (char*)y + (size_t)g.k0 * g.PQ * 2,
                         (int64_t)g.K * g.PQ, st);
    return check_launch();
  }
  const FwdPlan p = plan_fwd(g, desc->dtype);
  if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  char* base = (char*)ws;
  float* xt = (float*)(base + p.off_xt);
  float* yt = (float*)(base + p.off_yt);
  const size_t es = elem_size(desc->dtype);

  // x[N][C*H*W] -> x_t[C*H*W][Np]
  if (!input_ready)
    launch_transpose_in(desc->dtype, x, 0, (int64_t)g.C * g.HW, g.N, g.C * g.HW, xt, 0, g.Np, g.Np, 1,
                        xt - cs::ZERO_PAGE_FLOATS, st);
  const float* wmat;
  if (p.repitch) {
    float* wp = (float*)(base + p.off_w);
    const int blocks = (int)((((int64_t)g.Ks * p.ldw + 255) / 256 < 4096) ? ((int64_t)g.Ks * p.ldw + 255) / 256 : 4096);
    const char* wsrc = (const char*)w + (size_t)g.k0 * g.CRS * es;
    if (desc->dtype == CONV_F32)
      hipLaunchKernelGGL(cs::repitch_rows_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)wsrc,
                         (int64_t)g.CRS, g.Ks, g.CRS, wp, p.ldw);
    else
      hipLaunchKernelGGL(cs::repitch_rows_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st,
                         (const uint16_t*)wsrc, (int64_t)g.CRS, g.Ks, g.CRS, wp, p.ldw);
    wmat = wp;
  } else {
    wmat = (const float*)w + (size_t)g.k0 * g.CRS;
  }
  // three chunks more than needed: addresses are computed two chunks ahead and the table is read one further
  int* tab = (int*)(base + p.off_tab);
  const int entries = (p.nch + 4) * cs::BK;
  hipLaunchKernelGGL(cs::fwd_tap_table_kernel, dim3((entries + 255) / 256), dim3(256), 0, st, g, entries, tab);
  float* partial = (float*)(base + p.off_tail);
  probe.begin(st);
  rc = launch_fwd_gemm(g, needs_pad_checks(g), wmat, p.ldw, xt, tab, entries, yt, p.CT, p.nch, partial, st);
  probe.end(st);
  if (rc != CONV_OK) return rc;
  // y_t[Ks*P*Q][Np] -> y[n][k0*P*Q + ...]
  launch_transpose_out(desc->dtype, false, yt, g.Np, g.N, g.Ks * g.PQ,
                       (char*)y + (size_t)g.k0 * g.PQ * es, (int64_t)g.K * g.PQ, st);
  return check_launch();
}

}  // namespace

extern "C" {

int conv_fwd(const conv_desc_t* desc, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
             void* hip_stream) {
  return fwd_impl(desc, x, w, y, ws, ws_bytes, hip_stream, false);
}

// ---- forward pass for callers that cannot allocate: the workspace is a device array of the library ----
}  // extern "C"

namespace {

constexpr size_t kStaticScratchBytes = (size_t)CONV_NOALLOC_MAX_WORKSPACE;
// In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU (every GPU holds its own copy)
std::mutex g_scratch_mu;

// The device address of this GPU's copy of `scratch`, looked up once per device with that device current.
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CONV_ERR_LAUNCH;
  const std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return CONV_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return CONV_OK;
}

}  // namespace

extern "C" {

int conv_fwd_noalloc(const conv_desc_t* desc, const void* x, const void* w, void* y, void* hip_stream) {
  Geo g;
  const int rc = make_geo(desc, g);
  if (rc != CONV_OK) return rc;
  if (!x || !w || !y) return CONV_ERR_NULL;
  if (conv_workspace_bytes(desc, CONV_PASS_FWD) > kStaticScratchBytes) return CONV_ERR_WORKSPACE;
  if (g.Ks == 0) return CONV_OK;
  void* ws = nullptr;
  const int rs = static_scratch(&ws);
  if (rs != CONV_OK) return rs;
  // Every part of the workspace a kernel reads is written earlier in the same call (work copies, zero pages,
  // tap table, tail slots), so nothing has to be cleared between calls.
  return conv_fwd(desc, x, w, y, ws, kStaticScratchBytes, hip_stream);
}

int conv_bwd_data(const conv_desc_t* desc, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes,
                  void* hip_stream) {
  const Probe probe;
  Geo g;
  int rc = make_geo(desc, g);
  if (rc != CONV_OK) return rc;
  if (!dy || !w || !dx) return CONV_ERR_NULL;
  if (misaligned(dy, 16) || misaligned(w, 16) || misaligned(dx, 16)) return CONV_ERR_ALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t es = elem_size(desc->dtype);
  if (g.Ks == 0) {
    if (!desc->accumulate) {
      const int64_t count = (int64_t)g.N * g.C * g.HW;
      const int blocks = (int)((count + 255) / 256 < 8192 ? (count + 255) / 256 : 8192);
      if (desc->dtype == CONV_F32)
        hipLaunchKernelGGL(cs::fill_zero_kernel<float>, dim3(blocks), dim3(256), 0, st, (float*)dx, count);
      else
        hipLaunchKernelGGL(cs::fill_zero_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, (uint16_t*)dx, count);
      return check_launch();
    }
    return CONV_OK;
  }
  const PmPlan pm = plan_pm(g, desc->dtype);
  if (pm.ok_data) return pm_bwd_data(g, pm, desc->dtype, desc->accumulate != 0, dy, w, dx, ws, ws_bytes, st, probe);
  if (bf16_mfma_bwd_data_ok(g, desc->dtype)) {
    const BwdData16Plan p = plan_bwd_data16(g);
    if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
    char* base = (char*)ws;
    cs::bf16_t* dyp = (cs::bf16_t*)(base + p.off_dy);
    cs::bf16_t* wp = (cs::bf16_t*)(base + p.off_w);
    float* dxt = (float*)(base + p.off_dxt);
    int* perm = (int*)(base + p.off_perm);
    // per image: dy[n][k0..k1) as a Ks x PQ matrix -> dy_pqnk[pq][n][Ksp]; images N..Np-1 are zero
    launch_transpose_in(CONV_BF16, (const char*)dy + (size_t)g.k0 * g.PQ * 2, (int64_t)g.K * g.PQ, g.PQ, g.Ks, g.PQ,
                        dyp, p.Ksp, (int64_t)g.Np * p.Ksp, p.Ksp, g.Np, (float*)(base + p.off_dy - kZeroBytes), st,
                        true, g.N);
    // w[k][(c,rs)] -> w_rsck[rs][c][Ksp]: the slice's filter matrix transposed, rows re-ordered tap-major, zero past Ks
    launch_transpose_in(CONV_BF16, (const char*)w + (size_t)g.k0 * g.CRS * 2, 0, g.CRS, g.Ks, g.CRS, wp, 0, p.Ksp,
                        p.Ksp, 1, nullptr, st, true, -1, g.RS, g.C);
    const int MB = p.MB, CT = p.CT, bpt = p.wide ? 8 : 4;
    int* pre = (int*)(base + p.off_pre);
    float* partial = (float*)(base + p.off_tail);
    hipLaunchKernelGGL(cs::bwd_data_pixel_order_kernel, dim3(1), dim3(cs::po::THREADS), 0, st, g, perm,
                       (int*)(base + p.off_scratch), CT, p.Ksp / cs::BK16, bpt, p.run.enabled ? pre : (int*)nullptr);
    cs::bf16_t* zero = (cs::bf16_t*)(base + p.off_zero);
    hipLaunchKernelGGL(cs::fill_zero_kernel<uint16_t>, dim3(16), dim3(256), 0, st, zero, (int64_t)32 * p.Ksp + 64);
    const dim3 grid(p.run.enabled ? (p.run.nWg + 7) / 8 * 8 : cs::grid_dealt(MB, CT));
    if (p.wide) {
      const int lds = cs::SMEM2_BYTES + (g.RS + 3) * 36;   // stages + tap list + eight tap offsets per tap
      if ((rc = allow_big_lds(cs::bwd_data16_wide_gemm_kernel, lds)) != CONV_OK) return rc;
      probe.begin(st);
      hipLaunchKernelGGL(cs::bwd_data16_wide_gemm_kernel, grid, dim3(cs::NT2), lds, st, g, wp, p.Ksp, dyp, zero, perm, pre,
                         dxt, MB, CT, p.run, partial);
      if (p.run.enabled)
        hipLaunchKernelGGL(cs::bwd_data16_wide_fixup_kernel, dim3(CT * MB, 8), dim3(cs::NT2), 0, st, g, perm, pre, partial,
                           dxt, MB, CT, p.Ksp / cs::BK16, p.run.nRuns);
    } else {
      const int lds = cs::SMEM_BYTES + (g.RS + 3) * 20;
      if ((rc = allow_big_lds(cs::bwd_data16_gemm_kernel, lds)) != CONV_OK) return rc;
      probe.begin(st);
      hipLaunchKernelGGL(cs::bwd_data16_gemm_kernel, grid, dim3(cs::NT), lds, st, g, wp, p.Ksp, dyp, zero, perm, pre, dxt,
                         MB, CT, p.run, partial);
      if (p.run.enabled)
        hipLaunchKernelGGL(cs::bwd_data_fixup_kernel<2>, dim3(CT * MB, 4), dim3(cs::NT), 0, st, g, perm, pre, partial, dxt,
                           0, MB, CT, p.Ksp / cs::BK16, p.run.nRuns);
    }
    probe.end(st);
    launch_transpose_out(CONV_BF16, desc->accumulate != 0, dxt, g.Np, g.N, g.C * g.HW, dx, (int64_t)g.C * g.HW, st);
    return check_launch();
  }
  const BwdDataPlan p = plan_bwd_data(g);
  if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
  char* base = (char*)ws;
  float* dyt = (float*)(base + p.off_dyt);
  float* wt = (float*)(base + p.off_wt);
  float* dxt = (float*)(base + p.off_dxt);
  int* perm = (int*)(base + p.off_perm);

  if (p.scatter) {
    // dy[n][k0*PQ ..] -> dy_t[Ks*P*Q][Np]
    launch_transpose_in(desc->dtype, (const char*)dy + (size_t)g.k0 * g.PQ * es, 0, (int64_t)g.K * g.PQ, g.N,
                        g.Ks * g.PQ, dyt, 0, g.Np, g.Np, 1, dyt - cs::ZERO_PAGE_FLOATS, st);
    // T[(c,r,s)][p][q][n] = sum_k w'[(c,r,s)][k] * dy_t[k][p][q][n] is the forward kernel of a 1x1 layer
    // with Ks input channels, C*R*S kernels and dy_t as its input.
    Geo g1 = g;
    g1.C = g.Ks; g1.H = g.P; g1.W = g.Q; g1.K = g.CRS; g1.R = g1.S = 1; g1.sh = g1.sw = 1; g1.ph = g1.pw = 0;
    g1.k0 = 0; g1.Ks = g.CRS; g1.HW = g.PQ; g1.RS = 1; g1.CRS = g.Ks;
    float* T = (float*)(base + p.off_T);
    int* tab = (int*)(base + p.off_tab);
    // w[k][(c,r,s)] -> w'[(c,r,s)][Ksp], zero past Ks
    launch_transpose_in(desc->dtype, (const char*)w + (size_t)g.k0 * g.CRS * es, 0, g.CRS, g.Ks, g.CRS, wt, 0,
                        p.Ksp, p.Ksp, 1, nullptr, st);
    const int entries = (p.nch + 4) * cs::BK;
    hipLaunchKernelGGL(cs::fwd_tap_table_kernel, dim3((entries + 255) / 256), dim3(256), 0, st, g1, entries, tab);
    float* partial = (float*)(base + p.off_tail);
    probe.begin(st);
    rc = launch_fwd_gemm(g1, false, wt, p.Ksp, dyt, tab, entries, T, p.CT1, p.nch, partial, st);
    probe.end(st);
    if (rc != CONV_OK) return rc;
    const dim3 grid((g.C * g.HW + cs::COL2IM_ROWS - 1) / cs::COL2IM_ROWS, (g.N + 63) / 64);
    const bool acc = desc->accumulate != 0;
    if (desc->dtype == CONV_F32) {
      if (acc) hipLaunchKernelGGL((cs::col2im_out_kernel<float, true>), grid, dim3(256), 0, st, g, T, (float*)dx);
      else hipLaunchKernelGGL((cs::col2im_out_kernel<float, false>), grid, dim3(256), 0, st, g, T, (float*)dx);
    } else {
      if (acc) hipLaunchKernelGGL((cs::col2im_out_kernel<uint16_t, true>), grid, dim3(256), 0, st, g, T, (uint16_t*)dx);
      else hipLaunchKernelGGL((cs::col2im_out_kernel<uint16_t, false>), grid, dim3(256), 0, st, g, T, (uint16_t*)dx);
    }
    return check_launch();
  }
  // dy[n][k0*PQ ..] -> dy_t[k][P*Q + 1][Np]: one row left free after the P*Q pixels of every kernel.  That
  // pixel and the rows of kernels Ks .. Ksp-1 are cleared: taps that miss read the one, the reduction tail the other.
  const int64_t kPitch = (int64_t)(g.PQ + 1) * g.Np;
  launch_transpose_in(desc->dtype, (const char*)dy + (size_t)g.k0 * g.PQ * es, 0, (int64_t)g.K * g.PQ, g.N,
                      g.Ks * g.PQ, dyt, 0, g.Np, g.Np, 1, nullptr, st, false, -1, g.PQ);
  hipLaunchKernelGGL(cs::fill_zero_rows_kernel, dim3(std::min(1024, (g.Ks * g.Np + 255) / 256)), dim3(256), 0, st,
                     dyt + (int64_t)g.PQ * g.Np, kPitch, g.Ks, g.Np);
  if (p.Ksp > g.Ks)
    hipLaunchKernelGGL(cs::fill_zero_kernel<float>, dim3(1024), dim3(256), 0, st, dyt + (int64_t)g.Ks * kPitch,
                       (int64_t)(p.Ksp - g.Ks) * kPitch);
  // w[k][(c,rs)] -> w_t[rs][c][Ksp]: the slice's filter matrix transposed, its rows (c,rs) re-ordered tap-major,
  // zero past Ks.  A tap's C rows are then a dense C x Ksp matrix, contiguous along the reduction.
  launch_transpose_in(desc->dtype, (const char*)w + (size_t)g.k0 * g.CRS * es, 0, g.CRS, g.Ks, g.CRS, wt, 0, p.Ksp,
                      p.Ksp, 1, nullptr, st, false, -1, g.RS, g.C);
  int* pre = (int*)(base + p.off_pre);
  int* scratch = (int*)(base + p.off_scratch);
  float* partial = (float*)(base + p.off_tail);
  const int CT = (g.HW * g.NB + 3) / 4;
  const bool runs = (int64_t)CT * g.RS * p.nch < (int64_t)1 << 30;   // else the line would be too long for an int
  hipLaunchKernelGGL(cs::bwd_data_pixel_order_kernel, dim3(1), dim3(cs::po::THREADS), 0, st, g, perm, scratch, CT, p.nch,
                     4, runs ? pre : (int*)nullptr);
  // tiles + tap list + per-block tap offsets
  const int lds = cs::SMEM_BYTES + (g.RS + 3) * 20;
  // Channels in full row tiles first, then the half tile for a rest of at most 64 channels; both launches walk the
  // same line of column tiles and share the scratch slots (stream order keeps them apart).
  const RowSplit rs = split_rows(g.C, true);
  // one launch over `tiles` row tiles of shape mi from channel c0
  auto launch = [&](auto kern, auto fixup, int mi, int c0, int tiles) -> int {
    const int r = allow_big_lds(kern, lds);
    if (r != CONV_OK) return r;
    const cs::RunPlan rp = plan_runs(tiles, runs, 0, std::min(p.rounds, run_rounds(p.line, tiles)));
    hipLaunchKernelGGL(kern, dim3(rp.enabled ? (rp.nWg + 7) / 8 * 8 : cs::grid_dealt(tiles, CT)), dim3(cs::NT), lds, st, g,
                       wt, p.Ksp, dyt, perm, pre, dxt, c0, tiles, CT, rp, partial);
    if (rp.enabled)
      hipLaunchKernelGGL(fixup, dim3(CT * tiles, mi == 2 ? 4 : mi == 1 ? 2 : 3), dim3(cs::NT), 0, st, g, perm, pre, partial,
                         dxt, c0, tiles, CT, p.nch, rp.nRuns);
    return CONV_OK;
  };
  probe.begin(st);
  if (rs.full > 0) rc = launch(cs::bwd_data_gemm_kernel<2>, cs::bwd_data_fixup_kernel<2>, 2, 0, rs.full);
  if (rc == CONV_OK && rs.last == 1)
    rc = launch(cs::bwd_data_gemm_kernel<1>, cs::bwd_data_fixup_kernel<1>, 1, rs.full * cs::BM, 1);
  if (rc == CONV_OK && rs.last == 3)
    rc = launch(cs::bwd_data_gemm_kernel<3>, cs::bwd_data_fixup_kernel<3>, 3, rs.full * cs::BM, rs.nlast);
  if (rc != CONV_OK) return rc;
  probe.end(st);
  // dx_t[C*H*W][Np] -> dx[N][C*H*W]
  launch_transpose_out(desc->dtype, desc->accumulate != 0, dxt, g.Np, g.N, g.C * g.HW, dx, (int64_t)g.C * g.HW, st);
  return check_launch();
}

}  // extern "C"

namespace {

int bwd_weight_impl(const conv_desc_t* desc, const void* x, const void* dy, void* dw, void* ws, size_t ws_bytes,
                    void* hip_stream, bool input_ready) {
  const Probe probe;
  Geo g;
  int rc = make_geo(desc, g);
  if (rc != CONV_OK) return rc;
  if (!x || !dy || !dw) return CONV_ERR_NULL;
  if (misaligned(x, 16) || misaligned(dy, 16) || misaligned(dw, 16)) return CONV_ERR_ALIGN;
  if (g.Ks == 0) return CONV_OK;
  if (bf16_mfma_bwd_weight_ok(g, desc->dtype)) {
    const BwdWeight16Plan p = plan_bwd_weight16(g);
    if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    char* base = (char*)ws;
    cs::bf16_t* xt = (cs::bf16_t*)(base + p.off_xt);
    cs::bf16_t* dyt = (cs::bf16_t*)(base + p.off_dyt);
    float* dwslice = (float*)dw + (size_t)g.k0 * g.CRS;
    if (!input_ready)
      launch_transpose_in(CONV_BF16, x, 0, (int64_t)g.C * g.HW, g.N, g.C * g.HW, xt, 0, p.Np64, p.Np64, 1,
                          (float*)(base + p.off_xt - kZeroBytes), st, true);
    launch_transpose_in(CONV_BF16, (const char*)dy + (size_t)g.k0 * g.PQ * 2, 0, (int64_t)g.K * g.PQ, g.N,
                        g.Ks * g.PQ, dyt, 0, p.Np64, p.Np64, 1, nullptr, st, true);
    const bool pad16 = needs_pad_checks(g);
    const int64_t sliceElems = (int64_t)g.Ks * g.CRS;
    float* out = p.splits > 1 ? (float*)(base + p.off_part) : dwslice;
    float* partial = (float*)(base + p.off_tail);
    const dim3 grid(split_grid(p.MB * p.CT, p.splits, p.tail));
    auto launch = [&](auto kern, auto fixup, int threads, int lds, auto... fixArgs) -> int {
      const int r = allow_big_lds(kern, lds);
      if (r != CONV_OK) return r;
      probe.begin(st);
      hipLaunchKernelGGL(kern, grid, dim3(threads), lds, st, g, dyt, xt, p.Np64, out, sliceElems, p.MB, p.CT, p.nch,
                         p.chPerSplit, p.splits, p.tail, partial);
      if (p.tail.nTail > 0)
        hipLaunchKernelGGL(fixup, dim3(p.tail.nTail, threads / 64), dim3(threads), 0, st, g, partial, out, fixArgs..., p.MB,
                           p.CT, p.nch, p.tail);
      probe.end(st);
      return CONV_OK;
    };
    if (p.wide)
      rc = pad16 ? launch(cs::bwd_weight16_wide_gemm_kernel<true>, cs::bwd_weight16_wide_fixup_kernel, cs::NT2, cs::SMEM2_BYTES)
                 : launch(cs::bwd_weight16_wide_gemm_kernel<false>, cs::bwd_weight16_wide_fixup_kernel, cs::NT2, cs::SMEM2_BYTES);
    else
      rc = pad16 ? launch(cs::bwd_weight16_gemm_kernel<true>, cs::bwd_weight_tail_fixup_kernel<2>, cs::NT, cs::SMEM_BYTES, 0, 0)
                 : launch(cs::bwd_weight16_gemm_kernel<false>, cs::bwd_weight_tail_fixup_kernel<2>, cs::NT, cs::SMEM_BYTES, 0, 0);
    if (rc != CONV_OK) return rc;
    if (p.splits > 1) {
      const int blocks = (int)((sliceElems + 255) / 256 < 8192 ? (sliceElems + 255) / 256 : 8192);
      hipLaunchKernelGGL(cs::splitk_reduce_kernel, dim3(blocks), dim3(256), 0, st, out, sliceElems, p.splits,
                         dwslice, sliceElems);
    }
    return check_launch();
  }
  {
    const PmPlan pm = plan_pm(g, desc->dtype);
    if (pm.ok) return pm_bwd_weight(g, pm, x, dy, dw, ws, ws_bytes, (hipStream_t)hip_stream, probe, input_ready);
  }
  const BwdWeightPlan p = plan_bwd_weight(g);
  if ((rc = check_ws(ws, ws_bytes, p.total)) != CONV_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t es = elem_size(desc->dtype);
  char* base = (char*)ws;
  float* xt = (float*)(base + p.off_xt);
  float* dyt = (float*)(base + p.off_dyt);
  float* dwslice = (float*)dw + (size_t)g.k0 * g.CRS;

  if (!input_ready)
    launch_transpose_in(desc->dtype, x, 0, (int64_t)g.C * g.HW, g.N, g.C * g.HW, xt, 0, g.Np, g.Np, 1,
                        xt - cs::ZERO_PAGE_FLOATS, st);
  launch_transpose_in(desc->dtype, (const char*)dy + (size_t)g.k0 * g.PQ * es, 0, (int64_t)g.K * g.PQ, g.N,
                      g.Ks * g.PQ, dyt, 0, g.Np, g.Np, 1, nullptr, st);
  const bool pad = needs_pad_checks(g);
  float* scratch = (float*)(base + p.off_part);   // split partials or tail slots
  // One launch over `tiles` row tiles of shape mi (128, 64 or 96 rows) from row m0: the reduction split (partials,
  // then a sum in split order) or whole tiles with a shared tail.
  auto launch = [&](auto kern, auto fixup, int mi, int m0, int tiles) -> int {
    int rc2;
    if ((rc2 = allow_big_lds(kern, cs::SMEM_BYTES)) != CONV_OK) return rc2;
    const int rows = std::min(g.Ks - m0, tiles * (mi == 3 ? 96 : 64 * mi));
    const int splits = choose_splits((int64_t)tiles * p.CT, p.nch, true);
    cs::TailPlan tp;
    if (splits > 1) { tp.nFull = tiles * p.CT; tp.nTail = 0; tp.units = 1; tp.nTailWg = 0; }
    else tp = plan_tail(tiles * p.CT, p.nch);
    const int64_t stride = (int64_t)rows * g.CRS;
    float* out = splits > 1 ? scratch : dwslice;
    const int rowBase = splits > 1 ? m0 : 0;
    hipLaunchKernelGGL(kern, dim3(split_grid(tiles * p.CT, splits, tp)), dim3(cs::NT), cs::SMEM_BYTES, st, g, dyt, xt,
                       out, stride, m0, rowBase, tiles, p.CT, p.nch, splits, tp, scratch);
    if (tp.nTail > 0)
      hipLaunchKernelGGL(fixup, dim3(tp.nTail, mi == 2 ? 4 : mi == 1 ? 2 : 3), dim3(cs::NT), 0, st, g, scratch, out, m0,
                         rowBase, tiles, p.CT, p.nch, tp);
    if (splits > 1) {
      const int blocks = (int)((stride + 255) / 256 < 8192 ? (stride + 255) / 256 : 8192);
      hipLaunchKernelGGL(cs::splitk_reduce_kernel, dim3(blocks), dim3(256), 0, st, scratch, stride, splits,
                         dwslice + (int64_t)m0 * g.CRS, stride);
    }
    return CONV_OK;
  };
  const RowSplit rs = split_rows(g.Ks, true);
  probe.begin(st);
  if (rs.full > 0)
    rc = pad ? launch(cs::bwd_weight_gemm_kernel<true, 2>, cs::bwd_weight_tail_fixup_kernel<2>, 2, 0, rs.full)
             : launch(cs::bwd_weight_gemm_kernel<false, 2>, cs::bwd_weight_tail_fixup_kernel<2>, 2, 0, rs.full);
  if (rc == CONV_OK && rs.last == 1)
    rc = pad ? launch(cs::bwd_weight_gemm_kernel<true, 1>, cs::bwd_weight_tail_fixup_kernel<1>, 1, rs.full * cs::BM, 1)
             : launch(cs::bwd_weight_gemm_kernel<false, 1>, cs::bwd_weight_tail_fixup_kernel<1>, 1, rs.full * cs::BM, 1);
  if (rc == CONV_OK && rs.last == 3)
    rc = pad ? launch(cs::bwd_weight_gemm_kernel<true, 3>, cs::bwd_weight_tail_fixup_kernel<3>, 3, rs.full * cs::BM, rs.nlast)
             : launch(cs::bwd_weight_gemm_kernel<false, 3>, cs::bwd_weight_tail_fixup_kernel<3>, 3, rs.full * cs::BM, rs.nlast);
  probe.end(st);
  if (rc != CONV_OK) return rc;
  return check_launch();
}

}  // namespace

namespace cs_internal {
int conv_fwd_shared(const conv_desc_t* desc, const void* x, const void* w, void* y, void* ws, size_t ws_bytes,
                    void* hip_stream, int input_ready) {
  return fwd_impl(desc, x, w, y, ws, ws_bytes, hip_stream, input_ready != 0);
}
int conv_bwd_weight_shared(const conv_desc_t* desc, const void* x, const void* dy, void* dw, void* ws, size_t ws_bytes,
                           void* hip_stream, int input_ready) {
  return bwd_weight_impl(desc, x, dy, dw, ws, ws_bytes, hip_stream, input_ready != 0);
}
}  // namespace cs_internal

extern "C" {

int conv_bwd_weight(const conv_desc_t* desc, const void* x, const void* dy, void* dw, void* ws, size_t ws_bytes,
                    void* hip_stream) {
  return bwd_weight_impl(desc, x, dy, dw, ws, ws_bytes, hip_stream, false);
}

const char* conv_pass_path(const conv_desc_t* desc, int pass) {
  Geo g;
  if (make_geo(desc, g) != CONV_OK) return "invalid descriptor";
  const int dt = desc->dtype;
  const bool bf = dt == CONV_BF16;
  const PmPlan pm = plan_pm(g, dt);
  switch (pass) {
    case CONV_PASS_FWD:
      if (pm.ok && plan_pm16_fwd(g, pm, dt).ok)
        return "fwd16_pm_gemm_kernel: bf16 MFMA, pixel-major on a channels-last copy of x, y stored in place";
      if (pm.ok) return bf ? "fwd_pm_gemm_kernel: fp32 MFMA on operands converted from bf16, pixel-major, y stored in place"
                           : "fwd_pm_gemm_kernel: fp32 MFMA, pixel-major, y stored in place";
      if (bf16_mfma_fwd_ok(g, dt))
        return plan_fwd16(g).wide ? "fwd16_wide_gemm_kernel: bf16 MFMA, 256 x 256 tiles, batch-innermost work copies"
                                  : "fwd16_gemm_kernel: bf16 MFMA, batch-innermost work copies";
      return bf ? "fwd_gemm_kernel: fp32 MFMA on operands converted from bf16, batch-innermost work copies"
                : "fwd_gemm_kernel: fp32 MFMA, batch-innermost work copies";
    case CONV_PASS_BWD_DATA:
      if (pm.ok_data && plan_pm_bwd_data(g, dt).mfma16)
        return "bwd_data16_pm_gemm_kernel: bf16 MFMA, pixel-major T = w^T dy on a channels-last copy of dy, then col2im_pm_kernel";
      if (pm.ok_data)
        return bf ? "bwd_data_pm_gemm_kernel: fp32 MFMA on operands converted from bf16, pixel-major T = w^T dy, then col2im_pm_kernel"
                  : "bwd_data_pm_gemm_kernel: fp32 MFMA, pixel-major T = w^T dy read from dy in place, then col2im_pm_kernel";
      if (bf16_mfma_bwd_data_ok(g, dt))
        return plan_bwd_data16(g).wide
                   ? "bwd_data16_wide_gemm_kernel: bf16 MFMA, 256 x 256 tiles, per-pixel taps, batch-innermost work copies"
                   : "bwd_data16_gemm_kernel: bf16 MFMA, per-pixel taps, batch-innermost work copies";
      if (plan_bwd_data(g).scatter)
        return bf ? "fwd_gemm_kernel: fp32 MFMA on operands converted from bf16, T = w^T dy, then col2im_out_kernel"
                  : "fwd_gemm_kernel: fp32 MFMA, T = w^T dy on batch-innermost work copies, then col2im_out_kernel";
      return bf ? "bwd_data_gemm_kernel: fp32 MFMA on operands converted from bf16, per-pixel taps, batch-innermost work copies"
                : "bwd_data_gemm_kernel: fp32 MFMA, per-pixel taps, batch-innermost work copies";
    case CONV_PASS_BWD_WEIGHT:
      if (bf16_mfma_bwd_weight_ok(g, dt))
        return plan_bwd_weight16(g).wide ? "bwd_weight16_wide_gemm_kernel: bf16 MFMA, 256 x 256 tiles, batch-innermost work copies"
                                         : "bwd_weight16_gemm_kernel: bf16 MFMA, batch-innermost work copies";
      if (pm.ok) return "bwd_weight_pm_gemm_kernel: fp32 MFMA, pixel-major, dy read in place";
      return bf ? "bwd_weight_gemm_kernel: fp32 MFMA on operands converted from bf16, batch-innermost work copies"
                : "bwd_weight_gemm_kernel: fp32 MFMA, batch-innermost work copies";
    default: return "unknown pass";
  }
}

int conv_probe_next_call(void* start_event, void* stop_event) {
  tl_probe_start = (start_event && stop_event) ? (hipEvent_t)start_event : nullptr;
  tl_probe_stop = (start_event && stop_event) ? (hipEvent_t)stop_event : nullptr;
  return CONV_OK;
}

const char* conv_status_string(int status) {
  switch (status) {
    case CONV_OK: return "ok";
    case CONV_ERR_NULL: return "a required pointer is NULL";
    case CONV_ERR_SHAPE: return "invalid or unsupported tensor shape";
    case CONV_ERR_SLICE: return "kernel slice must satisfy 0 <= k0 <= k1 <= K";
    case CONV_ERR_DTYPE: return "unknown dtype";
    case CONV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CONV_ERR_LAUNCH: return "HIP launch failed";
    case CONV_ERR_ALIGN: return "tensor pointer is not 16-byte aligned";
    case CONV_ERR_PASS: return "unknown pass";
    case CONV_ERR_PARTITION: return "invalid times, device count or kernel bounds";
    default: return "unknown status";
  }
}

}  // extern "C"
