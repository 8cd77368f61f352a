// bfloat16 matrix-core passes: v_mfma_f32_32x32x16_bf16 with fp32 accumulation.
//
// In that instruction lane l supplies the eight consecutive reduction elements
// k = 8*(l/32) .. +7 of row (or column) l%32, i.e. 16 bytes.  So both operands are staged
// as col images (see conv_common.h): a tile row holds 64 reduction elements as eight
// 16-byte slots, and one 16-byte LDS read is one MFMA operand.  To make every operand
// contiguous along the reduction, each pass gets its own packed bf16 copies:
//
//   fwd        reduction (r,s,c):  w_krsc[Ks][R*S][Cp]          x_hwnc[H][W][Np][Cp]
//   bwd_data   reduction (tap,k):  w_rsck[R*S][C][Ksp]          dy_pqnk[P][Q][Np][Ksp]
//   bwd_weight reduction (pix,n):  dy_t[Ks][P*Q][Np64]          x_t[C][H][W][Np64]
//
// with Cp, Ksp, Np64 rounded up to 64 and zero filled, so a chunk (64 reduction elements)
// never needs a tail mask.  Tiles, column blocks, tap lists, XCD maps and epilogues are
// those of the fp32 kernels; outputs leave the kernels as fp32 (y_t, dx_t, dw).
#pragma once
#include "conv_common.h"
#include "gemm_kernels.h"

namespace cs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t bf16_t;                  // storage type of a bfloat16 element
constexpr int BK16 = 64;                  // reduction elements per chunk
constexpr int ZERO_PAGE_BF16 = ZERO_PAGE_FLOATS * 2;   // the zero page counted in bf16 elements

// 16-byte slot of a lane inside a chunk row of the col image, in bf16 elements (load i, lane l).
__device__ __forceinline__ int slot8(int l, int i) { return 8 * ((l & 7) ^ col_key(8 * i + (l >> 3))); }

struct Frag16 {
  f32x4 v[2];   // one MFMA operand (8 bf16) for each of the wavefront's two 32-wide blocks
};

// Operands of MFMA step j (0..3) of a chunk from a col image: logical slot 2*j + lane/32.
__device__ __forceinline__ void read_frag16(Frag16& f, const float* tile, int wbase, int lane, int j) {
  const int u = col_key(lane & 31), h = lane >> 5;
  const int slot = (wbase + (lane & 31)) * 8 + ((2 * j + h) ^ u);
  f.v[0] = *(const f32x4*)(tile + slot * 4);
  f.v[1] = *(const f32x4*)(tile + slot * 4 + 32 * 8 * 4);
}

__device__ __forceinline__ void mfma16_group(const Frag16& a, const Frag16& b, f32x16 (&acc)[2][2]) {
  const bf16x8 a0 = __builtin_bit_cast(bf16x8, a.v[0]), a1 = __builtin_bit_cast(bf16x8, a.v[1]);
  const bf16x8 b0 = __builtin_bit_cast(bf16x8, b.v[0]), b1 = __builtin_bit_cast(bf16x8, b.v[1]);
  acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
  acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
  acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
  acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
}

// Main loop: same driving protocol as the fp32 loop (begin / issue(0..3) / end, dummy loads
// past the last chunk) and the same rotation across the one barrier per chunk: after the
// barrier that publishes chunk ch a wavefront issues the DMA loads of chunk ch+1, runs steps
// 2,3 of chunk ch-1 from registers while the operand reads of steps 0,1 of chunk ch are in
// flight, then steps 0,1 of chunk ch while steps 2,3 are being read.
template <class LA, class LB>
__device__ __forceinline__ void gemm16_mainloop(LA& la, LB& lb, int ch_begin, int ch_end, float* smem,
                                                f32x16 (&acc)[2][2]) {
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wa = (wv >> 1) * 64, wb = (wv & 1) * 64;
  if (ch_begin >= ch_end) return;
  auto issue = [&](int ch, float* ta, float* tb, bool live) {
    la.begin(ch, live);
    lb.begin(ch, live);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      la.issue(i, ta + (wv * 4 + i) * 256);
      lb.issue(i, tb + (wv * 4 + i) * 256);
    }
    la.end();
    lb.end();
  };
  Frag16 a0, b0, a1, b1;
  issue(ch_begin, smem, smem + 2 * TILE_F, true);
  __syncthreads();
  read_frag16(a0, smem, wa, lane, 0);
  read_frag16(b0, smem + 2 * TILE_F, wb, lane, 0);
  read_frag16(a1, smem, wa, lane, 1);
  read_frag16(b1, smem + 2 * TILE_F, wb, lane, 1);
  issue(ch_begin + 1, smem + TILE_F, smem + 3 * TILE_F, ch_begin + 1 < ch_end);
  CS_FENCE();
  mfma16_group(a0, b0, acc);
  CS_FENCE();
  read_frag16(a0, smem, wa, lane, 2);
  read_frag16(b0, smem + 2 * TILE_F, wb, lane, 2);
  CS_FENCE();
  mfma16_group(a1, b1, acc);
  CS_FENCE();
  read_frag16(a1, smem, wa, lane, 3);
  read_frag16(b1, smem + 2 * TILE_F, wb, lane, 3);
  __syncthreads();
  int cur = TILE_F;
  for (int ch = ch_begin + 1; ch < ch_end; ++ch) {
    const float* As = smem + cur;
    const float* Bs = smem + 2 * TILE_F + cur;
    issue(ch + 1, smem + (cur ^ TILE_F), smem + 2 * TILE_F + (cur ^ TILE_F), ch + 1 < ch_end);
    CS_FENCE();
    mfma16_group(a0, b0, acc);  // step 2 of chunk ch-1
    CS_FENCE();
    read_frag16(a0, As, wa, lane, 0);
    read_frag16(b0, Bs, wb, lane, 0);
    CS_FENCE();
    mfma16_group(a1, b1, acc);  // step 3 of chunk ch-1
    CS_FENCE();
    read_frag16(a1, As, wa, lane, 1);
    read_frag16(b1, Bs, wb, lane, 1);
    CS_FENCE();
    mfma16_group(a0, b0, acc);  // step 0 of chunk ch
    CS_FENCE();
    read_frag16(a0, As, wa, lane, 2);
    read_frag16(b0, Bs, wb, lane, 2);
    CS_FENCE();
    mfma16_group(a1, b1, acc);  // step 1 of chunk ch
    CS_FENCE();
    read_frag16(a1, As, wa, lane, 3);
    read_frag16(b1, Bs, wb, lane, 3);
    __syncthreads();
    cur ^= TILE_F;
  }
  mfma16_group(a0, b0, acc);  // steps 2, 3 of the last chunk
  mfma16_group(a1, b1, acc);
}

// ------------------------------------------------------------- wide tiles ----
// 256 x 256 tiles for eight wavefronts (2 x 4, each 128 rows x 64 columns = 4 x 2 accumulator
// blocks): per MFMA a wavefront reads 0.75 operands from LDS instead of 1 and a workgroup stages
// half as many bytes, which is what limits the 128 x 128 loop at this instruction's rate.
// LDS holds two stages of two 32 KB col images (128 KB: one workgroup per compute unit).  The
// loaders are the same: wavefront wv stages rows (or column block) 32*wv .. 32*wv+31.
constexpr int NT2 = 512;
constexpr int BM2 = 256, BN2 = 256;
constexpr int TILE2_F = BM2 * BK16 / 2;         // floats of one operand stage (32 KB)
constexpr int SMEM2_BYTES = 4 * TILE2_F * 4;
constexpr int TAIL2_SLOT_FLOATS = 128 * NT2;    // one accumulator image of a wide tile (256 KB)

template <int NBLK>
struct Frag16N {
  f32x4 v[NBLK];
};
template <int NBLK>
__device__ __forceinline__ void read_frag16n(Frag16N<NBLK>& f, const float* tile, int wbase, int lane, int j) {
  const int u = col_key(lane & 31), h = lane >> 5;
  const int slot = (wbase + (lane & 31)) * 8 + ((2 * j + h) ^ u);
#pragma unroll
  for (int b = 0; b < NBLK; ++b) f.v[b] = *(const f32x4*)(tile + slot * 4 + b * (32 * 8 * 4));
}

__device__ __forceinline__ void mfma16_group_wide(const Frag16N<4>& a, const Frag16N<2>& b, f32x16 (&acc)[4][2]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const bf16x8 ai = __builtin_bit_cast(bf16x8, a.v[i]);
#pragma unroll
    for (int j = 0; j < 2; ++j)
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ai, __builtin_bit_cast(bf16x8, b.v[j]), acc[i][j], 0, 0, 0);
  }
}

// Same rotation across the one barrier per chunk as gemm16_mainloop.
template <class LA, class LB>
__device__ __forceinline__ void gemm16_mainloop_wide(LA& la, LB& lb, int ch_begin, int ch_end, float* smem,
                                                     f32x16 (&acc)[4][2]) {
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wa = (wv >> 2) * 128, wb = (wv & 3) * 64;
  if (ch_begin >= ch_end) return;
  auto issue = [&](int ch, float* ta, float* tb, bool live) {
    la.begin(ch, live);
    lb.begin(ch, live);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      la.issue(i, ta + (wv * 4 + i) * 256);
      lb.issue(i, tb + (wv * 4 + i) * 256);
    }
    la.end();
    lb.end();
  };
  Frag16N<4> a0, a1;
  Frag16N<2> b0, b1;
  float* const A = smem;
  float* const B = smem + 2 * TILE2_F;
  issue(ch_begin, A, B, true);
  __syncthreads();
  read_frag16n(a0, A, wa, lane, 0);
  read_frag16n(b0, B, wb, lane, 0);
  read_frag16n(a1, A, wa, lane, 1);
  read_frag16n(b1, B, wb, lane, 1);
  issue(ch_begin + 1, A + TILE2_F, B + TILE2_F, ch_begin + 1 < ch_end);
  CS_FENCE();
  mfma16_group_wide(a0, b0, acc);
  CS_FENCE();
  read_frag16n(a0, A, wa, lane, 2);
  read_frag16n(b0, B, wb, lane, 2);
  CS_FENCE();
  mfma16_group_wide(a1, b1, acc);
  CS_FENCE();
  read_frag16n(a1, A, wa, lane, 3);
  read_frag16n(b1, B, wb, lane, 3);
  __syncthreads();
  int cur = TILE2_F;
  for (int ch = ch_begin + 1; ch < ch_end; ++ch) {
    const float* As = A + cur;
    const float* Bs = B + cur;
    issue(ch + 1, A + (cur ^ TILE2_F), B + (cur ^ TILE2_F), ch + 1 < ch_end);
    CS_FENCE();
    mfma16_group_wide(a0, b0, acc);  // step 2 of chunk ch-1
    CS_FENCE();
    read_frag16n(a0, As, wa, lane, 0);
    read_frag16n(b0, Bs, wb, lane, 0);
    CS_FENCE();
    mfma16_group_wide(a1, b1, acc);  // step 3 of chunk ch-1
    CS_FENCE();
    read_frag16n(a1, As, wa, lane, 1);
    read_frag16n(b1, Bs, wb, lane, 1);
    CS_FENCE();
    mfma16_group_wide(a0, b0, acc);  // step 0 of chunk ch
    CS_FENCE();
    read_frag16n(a0, As, wa, lane, 2);
    read_frag16n(b0, Bs, wb, lane, 2);
    CS_FENCE();
    mfma16_group_wide(a1, b1, acc);  // step 1 of chunk ch
    CS_FENCE();
    read_frag16n(a1, As, wa, lane, 3);
    read_frag16n(b1, Bs, wb, lane, 3);
    __syncthreads();
    cur ^= TILE2_F;
  }
  mfma16_group_wide(a0, b0, acc);  // steps 2, 3 of the last chunk
  mfma16_group_wide(a1, b1, acc);
}

__device__ __forceinline__ void zero_acc_wide(f32x16 (&acc)[4][2]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
}

// Accumulator image of a wide tile: element e = (i*2+j)*16+v of thread t at [e*NT2 + t].
__device__ __forceinline__ void store_partial_wide(float* slot, const f32x16 (&acc)[4][2]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) slot[((i * 2 + j) * 16 + v) * NT2 + threadIdx.x] = acc[i][j][v];
}

// Sum of the scratch slots of tail tile tl, in run order, for accumulator block (bi,bj).
__device__ __forceinline__ void gather_partials_wide(const float* partial, const TailPlan& tp, int nch, int tl,
                                                     int bi, int bj, f32x16& acc) {
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  const int wfirst = (tl * nch) / tp.units;
  const int wlast = min(tp.nTailWg - 1, (tl * nch + nch - 1) / tp.units);
  for (int w = wfirst; w <= wlast; ++w) {
    const int slot = (w * tp.units) / nch == tl ? 0 : 1;
    const float* p = partial + (int64_t)(w * 2 + slot) * TAIL2_SLOT_FLOATS + (bi * 2 + bj) * 16 * NT2 + threadIdx.x;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] += p[v * NT2];
  }
}

// ------------------------------------------------------------------ forward ----
// A[m][kk] = w_krsc[m0+m][kk]: dense rows of R*S*Cp elements.  As in the fp32 kernels every
// load is "wave-uniform base + fixed per-lane byte offset", so the loop spends no vector
// instructions on addresses.
struct Fwd16LoadA {
  const char* tile;   // uniform: row m0
  const char* ub;
  unsigned off[4];
  __device__ Fwd16LoadA(const bf16_t* w, int64_t ldw, int m0, int Ks) : tile((const char*)(w + (int64_t)m0 * ldw)) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = min(32 * wv + 8 * i + (l >> 3), Ks - 1 - m0);  // rows past the slice repeat the last one
      off[i] = (unsigned)(m * ldw + slot8(l, i)) * 2u;
    }
  }
  __device__ __forceinline__ void begin(int ch, bool live) { ub = tile + (int64_t)(live ? ch : 0) * (BK16 * 2); }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {}
};

// B^T[(block,n)][kk] = x_hwnc[h0+r][w0+s][n][c]: chunk = (r, s, 64 channels); the pixel of
// a column block is uniform per wavefront (wavefront wv stages block wv of the tile), so a
// tap that falls into the padding switches the uniform base to a block of zeros.
template <int BPT = 4>   // column blocks per tile = wavefronts per workgroup
struct Fwd16LoadB {
  const char* x;        // uniform: x_hwnc at the block's images
  const char* zero;     // uniform: 32 rows of Cp zeros
  const char* ub;
  unsigned off[4];
  int h0, w0, H, W, S, R, ncc;
  int64_t pixBytes;     // one pixel: Np * Cp elements
  int r, s, cc;         // uniform walk over the next chunk to issue
  __device__ Fwd16LoadB(const Geo& g, const bf16_t* x_, const bf16_t* zero_, int Cp, int ct, int ch0)
      : zero((const char*)zero_) {
    const int l = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gcb = ct * BPT + wv < g.PQ * g.NB ? ct * BPT + wv : 0;   // blocks past the end: computed, never stored
    const int pix = gcb / g.NB, nb = gcb - pix * g.NB;
    const int p = pix / g.Q, q = pix - p * g.Q;
    h0 = p * g.sh - g.ph;
    w0 = q * g.sw - g.pw;
    H = g.H; W = g.W; S = g.S; R = g.R;
    pixBytes = (int64_t)g.Np * Cp * 2;
    x = (const char*)(x_ + (int64_t)nb * 32 * Cp);
    ncc = Cp / BK16;
#pragma unroll
    for (int i = 0; i < 4; ++i) off[i] = (unsigned)((8 * i + (l >> 3)) * Cp + slot8(l, i)) * 2u;
    const int tap = ch0 / ncc;
    cc = ch0 - tap * ncc;
    r = tap / S;
    s = tap - r * S;
  }
  __device__ __forceinline__ void begin(int, bool live) {
    const int hh = h0 + r, vv = w0 + s;
    const bool ok = live & ((unsigned)hh < (unsigned)H) & ((unsigned)vv < (unsigned)W);
    ub = ok ? x + (hh * W + vv) * pixBytes + cc * (BK16 * 2) : zero;
  }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {   // branch-free carry over (cc, s, r)
    ++cc;
    const int c1 = cc == ncc;
    cc = c1 ? 0 : cc;
    s += c1;
    const int c2 = s == S;
    s = c2 ? 0 : s;
    r += c2;
  }
};

__global__ __launch_bounds__(NT) void fwd16_gemm_kernel(Geo g, const bf16_t* __restrict__ w, int Cp,
                                                        const bf16_t* __restrict__ x,
                                                        const bf16_t* __restrict__ zero, float* __restrict__ yt,
                                                        int MB, int CT, int nch, TailPlan tp,
                                                        float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  for_each_segment(tp, nch, [&](int L, int cb, int ce, bool direct, int slot) {
    int mb, ct;
    tile_from_line(L, MB, CT, mb, ct);
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    Fwd16LoadA la(w, (int64_t)g.RS * Cp, mb * BM, g.Ks);
    Fwd16LoadB<4> lb(g, x, zero, Cp, ct, cb);
    gemm16_mainloop(la, lb, cb, ce, smem, acc);
    if (direct) fwd_store_tile<2>(g, yt, mb * BM, ct, acc);
    else store_partial<2>(partial + (int64_t)slot * TAIL_SLOT_FLOATS, acc);
  });
}

// Accumulator block (i,j) of a wide tile: 32 kernels x 32 images of one pixel.
__device__ __forceinline__ void fwd16_wide_store_block(const Geo& g, float* __restrict__ yt, int m0, int ct, int i, int j,
                                                       const f32x16& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int gcb = ct * 8 + (wave & 3) * 2 + j;
  if (gcb >= g.PQ * g.NB) return;
  const int pix = gcb / g.NB, nb = gcb - pix * g.NB;
  const int n = nb * 32 + (lane & 31);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + (wave >> 2) * 128 + i * 32 + acc_row(v, lane);
    if (m < g.Ks) yt[((int64_t)m * g.PQ + pix) * g.Np + n] = acc[v];
  }
}

// Forward pass on wide tiles: MB row tiles of 256 kernels, CT column tiles of eight blocks.
__global__ __launch_bounds__(NT2) void fwd16_wide_gemm_kernel(Geo g, const bf16_t* __restrict__ w, int Cp,
                                                              const bf16_t* __restrict__ x,
                                                              const bf16_t* __restrict__ zero, float* __restrict__ yt,
                                                              int MB, int CT, int nch, TailPlan tp,
                                                              float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  for_each_segment(tp, nch, [&](int L, int cb, int ce, bool direct, int slot) {
    int mb, ct;
    tile_from_line(L, MB, CT, mb, ct);
    f32x16 acc[4][2];
    zero_acc_wide(acc);
    Fwd16LoadA la(w, (int64_t)g.RS * Cp, mb * BM2, g.Ks);
    Fwd16LoadB<8> lb(g, x, zero, Cp, ct, cb);
    gemm16_mainloop_wide(la, lb, cb, ce, smem, acc);
    if (direct) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) fwd16_wide_store_block(g, yt, mb * BM2, ct, i, j, acc[i][j]);
    } else {
      store_partial_wide(partial + (int64_t)slot * TAIL2_SLOT_FLOATS, acc);
    }
  });
}

// grid = (nTail, 8): one workgroup per tail tile and accumulator block.
__global__ __launch_bounds__(NT2) void fwd16_wide_fixup_kernel(Geo g, const float* __restrict__ partial,
                                                               float* __restrict__ yt, int MB, int CT, int nch,
                                                               TailPlan tp) {
  const int bi = blockIdx.y >> 1, bj = blockIdx.y & 1;
  f32x16 acc;
  gather_partials_wide(partial, tp, nch, blockIdx.x, bi, bj, acc);
  int mb, ct;
  tile_from_line(tp.nFull + blockIdx.x, MB, CT, mb, ct);
  fwd16_wide_store_block(g, yt, mb * BM2, ct, bi, bj, acc);
}

// ----------------------------------------------------------- input gradient ----
// A[c][kk] = w_rsck[tap][c][k]: chunk = (tap, 64 kernels).
struct BwdData16LoadA {
  const char* wt;     // uniform: channel m0 of tap 0
  const char* ub;
  const int* taps;
  unsigned off[4];
  unsigned tapBytes;
  int S, tap;         // tap of walk.ti, fetched one call ahead (uniform, held in a vector register)
  TapWalk walk;
  __device__ BwdData16LoadA(const Geo& g, const bf16_t* wt_, int Ksp, int m0, const int* taps_, int nkc_, int ch0)
      : wt((const char*)(wt_ + (int64_t)m0 * Ksp)), taps(taps_), tapBytes((unsigned)g.C * (unsigned)Ksp * 2u), S(g.S),
        walk(nkc_, ch0) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = min(32 * wv + 8 * i + (l >> 3), g.C - 1 - m0);   // rows past C repeat the last one
      off[i] = (unsigned)(c * Ksp + slot8(l, i)) * 2u;
    }
    const int e = taps[walk.ti];
    tap = (e >> 16) * S + (e & 0xffff);
  }
  __device__ __forceinline__ void begin(int, bool live) {
    const unsigned t = (unsigned)__builtin_amdgcn_readfirstlane(tap);
    ub = wt + (live ? t * tapBytes + (unsigned)walk.kc * (BK16 * 2u) : 0u);
  }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {
    walk.next();
    const int e = taps[walk.ti];
    tap = (e >> 16) * S + (e & 0xffff);
  }
};

// B^T[(block,n)][kk] = dy_pqnk[p][q][n][k] with (p,q) the output pixel the current tap maps
// the block's input pixel to (from the per-tile LDS table; uniform per wavefront), or a block
// of zeros if there is none.
template <int BPT = 4>   // column blocks per tile = wavefronts per workgroup
struct BwdData16LoadB {
  const char* dy;     // uniform
  const char* zero;   // uniform: 32 rows of Ksp zeros
  const char* ub;
  const int* tapoff;
  unsigned off[4];
  int toff, wvb;      // toff: element offset of the block's 32 images at the tap's output pixel, or -1
  TapWalk walk;
  __device__ BwdData16LoadB(const bf16_t* dy_, const bf16_t* zero_, int Ksp, const int* tapoff_, int nkc_, int ch0)
      : dy((const char*)dy_), zero((const char*)zero_), tapoff(tapoff_), walk(nkc_, ch0) {
    const int l = threadIdx.x & 63;
    wvb = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int i = 0; i < 4; ++i) off[i] = (unsigned)((8 * i + (l >> 3)) * Ksp + slot8(l, i)) * 2u;
    toff = tapoff[walk.ti * BPT + wvb];
  }
  __device__ __forceinline__ void begin(int, bool live) {
    const int t = __builtin_amdgcn_readfirstlane(toff);
    ub = (live & (t >= 0)) ? dy + ((unsigned)t * 2u + (unsigned)walk.kc * (BK16 * 2u)) : zero;
  }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {
    walk.next();
    toff = tapoff[walk.ti * BPT + wvb];
  }
};

// Tiles, runs and scratch slots as in the fp32 kernel (RunPlan); the fp32 fix-up kernel serves both.
__global__ __launch_bounds__(NT) void bwd_data16_gemm_kernel(Geo g, const bf16_t* __restrict__ wt, int Ksp,
                                                             const bf16_t* __restrict__ dy,
                                                             const bf16_t* __restrict__ zero,
                                                             const int* __restrict__ perm,
                                                             const int* __restrict__ pre,
                                                             float* __restrict__ dxt, int MB, int CT, RunPlan rp,
                                                             float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  int* s_taps = (int*)(smem + 4 * TILE_F);     // [RS + 3]
  int* s_tapoff = s_taps + g.RS + 3;           // [RS + 3][4]
  __shared__ int s_ntaps;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nkc = Ksp / BK16;

  auto segment = [&](int mb, int ct, int c0, int c1, bool direct, int slot) {
    if (wave == 0) {   // tap list of the tile, as in the fp32 kernel; offsets are into dy_pqnk
      int hp[4], vp[4], nbo[4];
      bool ok[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int gcb = ct * 4 + j;
        ok[j] = gcb < g.HW * g.NB;
        const int sp = ok[j] ? gcb / g.NB : 0;
        const int px = perm[sp];
        nbo[j] = ok[j] ? (gcb - sp * g.NB) * 32 * Ksp : 0;
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
          offs[j] = hit ? (p * g.Q + q) * g.Np * Ksp + nbo[j] : -1;
          any |= hit;
        }
        const unsigned long long mask = __ballot(any);
        if (any) {
          const int pos = cnt + __popcll(mask & ((1ull << lane) - 1ull));
          s_taps[pos] = (rr << 16) | ss;
#pragma unroll
          for (int j = 0; j < 4; ++j) s_tapoff[pos * 4 + j] = offs[j];
        }
        cnt += __popcll(mask);
      }
      if (lane < 12) s_tapoff[cnt * 4 + lane] = -1;
      if (lane < 3) s_taps[cnt + lane] = 0;
      if (lane == 0) s_ntaps = cnt;
    }
    __syncthreads();
    const int nchunks = s_ntaps * nkc;
    const int cb = min(c0, nchunks), ce = min(c1, nchunks);
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    BwdData16LoadA la(g, wt, Ksp, mb * BM, s_taps, nkc, cb);
    BwdData16LoadB<4> lb(dy, zero, Ksp, s_tapoff, nkc, cb);
    gemm16_mainloop(la, lb, cb, ce, smem, acc);
    if (direct) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 2; ++i) bwd_data_store_block<2>(g, dxt, perm, mb * BM, ct, i, j, acc[i][j]);
    } else {
      store_partial<2>(partial + (int64_t)slot * TAIL_SLOT_FLOATS, acc);
    }
    __syncthreads();   // the next segment rewrites the tap list
  };

  if (!rp.enabled) {
    int mb, ct;
    if (!tile_dealt(blockIdx.x, MB, CT, mb, ct)) return;
    segment(mb, ct, 0, 0x7fffffff, true, 0);
    return;
  }
  const int wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  if (wg >= rp.nWg) return;
  const int run = wg / MB, mb = wg - run * MB;
  const int total = pre[CT], units = run_units(total, nkc, rp.nRuns);
  if ((int64_t)run * units >= total) return;
  int pos = run * units;
  const int end = min(pos + units, total);
  int ct = 0;   // the tile that holds pos: pre[ct] <= pos < pre[ct+1]
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

// Accumulator block (i,j) of a wide input-gradient tile: 32 channels x 32 images of one pixel.
__device__ __forceinline__ void bwd_data16_wide_store_block(const Geo& g, float* __restrict__ dxt,
                                                            const int* __restrict__ perm, int m0, int ct, int i, int j,
                                                            const f32x16& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // m0 does not change from one segment of a run to the next; the opaque copy keeps the row addresses from being
  // computed once in front of the run and held in registers across the main loop.
  asm volatile("" : "+s"(m0));
  const int gcb = ct * 8 + (wave & 3) * 2 + j;
  if (gcb >= g.HW * g.NB) return;
  const int sp = gcb / g.NB, nb = gcb - sp * g.NB;
  const int px = perm[sp];
  const int n = nb * 32 + (lane & 31);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int c = m0 + (wave >> 2) * 128 + i * 32 + acc_row(v, lane);
    if (c < g.C) dxt[((int64_t)c * g.HW + px) * g.Np + n] = acc[v];
  }
}

// Input gradient on wide tiles: MB row tiles of 256 channels, CT column tiles of eight blocks (pre, when the runs
// are enabled, must have been measured for tiles of eight blocks).  LDS behind the stages: tap list [RS + 3] and
// per-block offsets [RS + 3][8].
__global__ __launch_bounds__(NT2) void bwd_data16_wide_gemm_kernel(Geo g, const bf16_t* __restrict__ wt, int Ksp,
                                                                   const bf16_t* __restrict__ dy,
                                                                   const bf16_t* __restrict__ zero,
                                                                   const int* __restrict__ perm,
                                                                   const int* __restrict__ pre,
                                                                   float* __restrict__ dxt, int MB, int CT,
                                                                   RunPlan rp, float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  int* s_taps = (int*)(smem + 4 * TILE2_F);    // [RS + 3]
  int* s_tapoff = s_taps + g.RS + 3;           // [RS + 3][8]
  __shared__ int s_ntaps;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nkc = Ksp / BK16;

  auto segment = [&](int mb, int ct, int c0, int c1, bool direct, int slot) {
    if (wave == 0) {   // tap list of the tile: the taps that reach any of its (at most eight) pixels
      int hp[8], vp[8], nbo[8];
      bool ok[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int gcb = ct * 8 + j;
        ok[j] = gcb < g.HW * g.NB;
        const int sp = ok[j] ? gcb / g.NB : 0;
        const int px = perm[sp];
        nbo[j] = ok[j] ? (gcb - sp * g.NB) * 32 * Ksp : 0;
        hp[j] = px / g.W + g.ph;
        vp[j] = px % g.W + g.pw;
      }
      int cnt = 0;
      for (int b = 0; b < g.RS; b += 64) {
        const int tp = b + lane;
        const int rr = tp / g.S, ss = tp - rr * g.S;
        bool any = false;
        int offs[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int hr = hp[j] - rr, vs = vp[j] - ss;
          const int p = hr / g.sh, q = vs / g.sw;
          const bool hit = tp < g.RS && ok[j] && hr >= 0 && vs >= 0 && p * g.sh == hr && q * g.sw == vs &&
                           p < g.P && q < g.Q;
          offs[j] = hit ? (p * g.Q + q) * g.Np * Ksp + nbo[j] : -1;
          any |= hit;
        }
        const unsigned long long mask = __ballot(any);
        if (any) {
          const int pos = cnt + __popcll(mask & ((1ull << lane) - 1ull));
          s_taps[pos] = (rr << 16) | ss;
#pragma unroll
          for (int j = 0; j < 8; ++j) s_tapoff[pos * 8 + j] = offs[j];
        }
        cnt += __popcll(mask);
      }
      if (lane < 24) s_tapoff[cnt * 8 + lane] = -1;   // the loaders run up to three entries past the list
      if (lane < 3) s_taps[cnt + lane] = 0;
      if (lane == 0) s_ntaps = cnt;
    }
    __syncthreads();
    const int nchunks = s_ntaps * nkc;
    const int cb = min(c0, nchunks), ce = min(c1, nchunks);
    f32x16 acc[4][2];
    zero_acc_wide(acc);
    BwdData16LoadA la(g, wt, Ksp, mb * BM2, s_taps, nkc, cb);
    BwdData16LoadB<8> lb(dy, zero, Ksp, s_tapoff, nkc, cb);
    gemm16_mainloop_wide(la, lb, cb, ce, smem, acc);
    if (direct) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) bwd_data16_wide_store_block(g, dxt, perm, mb * BM2, ct, i, j, acc[i][j]);
    } else {
      store_partial_wide(partial + (int64_t)slot * TAIL2_SLOT_FLOATS, acc);
    }
    __syncthreads();   // the next segment rewrites the tap list
  };

  if (!rp.enabled) {
    int mb, ct;
    if (!tile_dealt(blockIdx.x, MB, CT, mb, ct)) return;
    segment(mb, ct, 0, 0x7fffffff, true, 0);
    return;
  }
  const int wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  if (wg >= rp.nWg) return;
  const int run = wg / MB, mb = wg - run * MB;
  const int total = pre[CT], units = run_units(total, nkc, rp.nRuns);
  if ((int64_t)run * units >= total) return;
  int pos = run * units;
  const int end = min(pos + units, total);
  int ct = 0;   // the tile that holds pos: pre[ct] <= pos < pre[ct+1]
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

// Adds up the scratch slots of every wide tile that was cut by a run boundary.  grid = (CT*MB, 8).
__global__ __launch_bounds__(NT2) void bwd_data16_wide_fixup_kernel(Geo g, const int* __restrict__ perm,
                                                                    const int* __restrict__ pre,
                                                                    const float* __restrict__ partial,
                                                                    float* __restrict__ dxt, int MB, int CT, int nkc,
                                                                    int nRuns) {
  const int ct = blockIdx.x / MB, mb = blockIdx.x - ct * MB;
  const int units = run_units(pre[CT], nkc, nRuns);
  const int a = pre[ct], b = pre[ct + 1];   // the tile's stretch of the line
  const int r0 = a / units, r1 = (b - 1) / units;
  if (r0 == r1) return;   // inside one run: stored directly
  const int bi = blockIdx.y >> 1, bj = blockIdx.y & 1;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  for (int r = r0; r <= r1; ++r) {
    const int slot = r * units >= a ? 0 : 1;   // a run that starts inside the tile used its first slot
    const float* p = partial + (int64_t)((r * MB + mb) * 2 + slot) * TAIL2_SLOT_FLOATS + (bi * 2 + bj) * 16 * NT2 + threadIdx.x;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] += p[v * NT2];
  }
  bwd_data16_wide_store_block(g, dxt, perm, mb * BM2, ct, bi, bj, acc);
}

// ---------------------------------------------------------- weight gradient ----
// A[k][kk] = dy_t[k][pix][n]: dense rows of P*Q*Np64 elements; chunk = 64 images of one pixel.
struct BwdWeight16LoadA {
  const char* tile;
  const char* ub;
  unsigned off[4];
  __device__ BwdWeight16LoadA(const bf16_t* dyt, int64_t ld, int m0, int Ks) : tile((const char*)(dyt + (int64_t)m0 * ld)) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = min(32 * wv + 8 * i + (l >> 3), Ks - 1 - m0);
      off[i] = (unsigned)(m * ld + slot8(l, i)) * 2u;
    }
  }
  __device__ __forceinline__ void begin(int ch, bool live) { ub = tile + (int64_t)(live ? ch : 0) * (BK16 * 2); }
  __device__ __forceinline__ void issue(int i, float* dst) { dma16_uv(ub, off[i], dst); }
  __device__ __forceinline__ void end() {}
};

// B^T[(c,r,s)][kk] = x_t[c][p*sh-ph+r][q*sw-pw+s][n]; zero where the tap is in the padding
// (PAD: the base is the zero page in front of x_t and a lane whose tap is outside reads it).
template <bool PAD>
struct BwdWeight16LoadB {
  const char* xt;       // uniform; PAD: the zero page ZERO_PAGE_BF16 elements in front of x_t
  const char* ub;
  unsigned coff[4];
  int rj[4], sj[4];
  int NB64, Q, sh, sw, ph, pw, H, W, Np64;
  int p, q, nb;
  int h0, v0;
  unsigned uoff;
  __device__ BwdWeight16LoadB(const Geo& g, const bf16_t* xt_, int Np64_, int j0, int ch0)
      : xt(PAD ? opaque_uniform(xt_ - ZERO_PAGE_BF16) : (const char*)xt_) {
    const int l = threadIdx.x & 63, wv = threadIdx.x >> 6;
    Np64 = Np64_; NB64 = Np64_ / BK16; Q = g.Q; sh = g.sh; sw = g.sw; ph = g.ph; pw = g.pw; H = g.H; W = g.W;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int j = j0 + 32 * wv + 8 * i + (l >> 3);
      const int jj = j < g.CRS ? j : 0;
      const int c = jj / g.RS, rs = jj - c * g.RS;
      rj[i] = rs / g.S;
      sj[i] = rs - rj[i] * g.S;
      coff[i] = (unsigned)(c * g.HW * Np64 + (rj[i] * g.W + sj[i]) * Np64 + slot8(l, i) + (PAD ? ZERO_PAGE_BF16 : 0)) * 2u;
    }
    const int pix = ch0 / NB64;
    nb = ch0 - pix * NB64;
    p = pix / Q;
    q = pix - p * Q;
  }
  __device__ __forceinline__ void begin(int, bool live) {
    h0 = live ? p * sh - ph : 0;
    v0 = live ? q * sw - pw : 0;
    const int u = (h0 * W + v0) * Np64 + (live ? nb * BK16 : 0);
    if (PAD) uoff = (unsigned)u * 2u;
    else ub = xt + (int64_t)u * 2;
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
  __device__ __forceinline__ void end() {
    ++nb;
    const int cq = nb == NB64;
    nb = cq ? 0 : nb;
    q += cq;
    const int cp = q == Q;
    q = cp ? 0 : q;
    p += cp;
  }
};

template <bool PAD>
__global__ __launch_bounds__(NT) void bwd_weight16_gemm_kernel(Geo g, const bf16_t* __restrict__ dyt,
                                                               const bf16_t* __restrict__ xt, int Np64,
                                                               float* __restrict__ out, int64_t splitStride,
                                                               int MB, int CT, int nch, int chPerSplit,
                                                               int splits, TailPlan tp, float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  // split mode: workgroup -> (tile, split) as in the fp32 kernel; a split is a block of chPerSplit chunks
  int z = 0, Lsplit = 0;
  if (splits > 1) {
    const int tiles = MB * CT;
    int item;
    if (!line_contiguous(blockIdx.x, tiles * splits, item)) return;
    z = item / tiles;
    Lsplit = item - z * tiles;
  }
  const int ch0 = z * chPerSplit;
  const int ch1 = min(nch, ch0 + chPerSplit);
  float* o = out + (int64_t)z * splitStride;
  auto compute = [&](int L, int cb, int ce, bool direct, int slot) __attribute__((always_inline)) {
    int mb, ct;
    tile_from_line(L, MB, CT, mb, ct);
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    BwdWeight16LoadA la(dyt, (int64_t)g.PQ * Np64, mb * BM, g.Ks);
    BwdWeight16LoadB<PAD> lb(g, xt, Np64, ct * BN, cb);
    gemm16_mainloop(la, lb, cb, ce, smem, acc);
    if (direct) bwd_weight_store_tile<2>(g, o, mb * BM, 0, ct, acc);
    else store_partial<2>(partial + (int64_t)slot * TAIL_SLOT_FLOATS, acc);
  };
  if (splits > 1) {
    compute(Lsplit, ch0, ch1, true, 0);
    return;
  }
  for_each_segment(tp, nch, compute);
}

// Accumulator block (i,j) of a wide weight-gradient tile: 32 kernels x 32 filter elements.
__device__ __forceinline__ void bwd_weight16_wide_store_block(const Geo& g, float* __restrict__ o, int m0, int ct, int i,
                                                              int j, const f32x16& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = ct * BN2 + (wave & 3) * 64 + j * 32 + (lane & 31);
  if (col >= g.CRS) return;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int m = m0 + (wave >> 2) * 128 + i * 32 + acc_row(v, lane);
    if (m < g.Ks) o[(int64_t)m * g.CRS + col] = acc[v];
  }
}

// Weight gradient on wide tiles; splits, tail plan and outputs as in bwd_weight16_gemm_kernel.
template <bool PAD>
__global__ __launch_bounds__(NT2) void bwd_weight16_wide_gemm_kernel(Geo g, const bf16_t* __restrict__ dyt,
                                                                     const bf16_t* __restrict__ xt, int Np64,
                                                                     float* __restrict__ out, int64_t splitStride,
                                                                     int MB, int CT, int nch, int chPerSplit,
                                                                     int splits, TailPlan tp,
                                                                     float* __restrict__ partial) {
  extern __shared__ __align__(16) float smem[];
  int z = 0, Lsplit = 0;
  if (splits > 1) {
    const int tiles = MB * CT;
    int item;
    if (!line_contiguous(blockIdx.x, tiles * splits, item)) return;
    z = item / tiles;
    Lsplit = item - z * tiles;
  }
  const int ch0 = z * chPerSplit;
  const int ch1 = min(nch, ch0 + chPerSplit);
  float* o = out + (int64_t)z * splitStride;
  auto compute = [&](int L, int cb, int ce, bool direct, int slot) __attribute__((always_inline)) {
    int mb, ct;
    tile_from_line(L, MB, CT, mb, ct);
    f32x16 acc[4][2];
    zero_acc_wide(acc);
    BwdWeight16LoadA la(dyt, (int64_t)g.PQ * Np64, mb * BM2, g.Ks);
    BwdWeight16LoadB<PAD> lb(g, xt, Np64, ct * BN2, cb);
    gemm16_mainloop_wide(la, lb, cb, ce, smem, acc);
    if (direct) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) bwd_weight16_wide_store_block(g, o, mb * BM2, ct, i, j, acc[i][j]);
    } else {
      store_partial_wide(partial + (int64_t)slot * TAIL2_SLOT_FLOATS, acc);
    }
  };
  if (splits > 1) {
    compute(Lsplit, ch0, ch1, true, 0);
    return;
  }
  for_each_segment(tp, nch, compute);
}

// grid = (nTail, 8)
__global__ __launch_bounds__(NT2) void bwd_weight16_wide_fixup_kernel(Geo g, const float* __restrict__ partial,
                                                                      float* __restrict__ out, int MB, int CT, int nch,
                                                                      TailPlan tp) {
  const int bi = blockIdx.y >> 1, bj = blockIdx.y & 1;
  f32x16 acc;
  gather_partials_wide(partial, tp, nch, blockIdx.x, bi, bj, acc);
  int mb, ct;
  tile_from_line(tp.nFull + blockIdx.x, MB, CT, mb, ct);
  bwd_weight16_wide_store_block(g, out, mb * BM2, ct, bi, bj, acc);
}

}  // namespace cs
