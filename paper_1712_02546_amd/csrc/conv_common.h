// Shared device-side definitions for the gfx950 convolution kernels.
//
// Internal data layout ("batch-innermost"): every tensor the matrix-core kernels
// touch is first re-laid with the image index n as the fastest dimension, padded
// with zeros to Np = 32*ceil(N/32):
//     x_t [C][H][W][Np]     y_t / dy_t [Ks][P][Q][Np]     dx_t [C][H][W][Np]
// A 32-lane MFMA column block is then "32 images at one pixel": every operand
// row is a dense, 128-byte-aligned run, padding and stride decide per block (not
// per element) whether a filter tap contributes, and the input-gradient pass
// visits only the taps that really reach a pixel (no work on padded zeros).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "geo.h"

namespace cs {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int NT = 256;             // threads per workgroup: 4 wavefronts in a 2x2 grid
constexpr int BM = 128;             // tile rows  (GEMM M)
constexpr int BN = 128;             // tile cols  (GEMM N) = 4 column blocks of 32
constexpr int BK = 32;              // reduction elements per staged chunk
constexpr int TILE_F = BM * BK;     // floats of one operand tile in LDS (16 KB)
constexpr int SMEM_BYTES = 4 * TILE_F * 4;  // A and B, two stages each: 64 KB
constexpr int ZERO_PAGE_FLOATS = 256;       // zero-filled scratch that masked lanes load from

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}

// Round-to-nearest-even fp32 -> bfloat16; NaN stays NaN (quiet).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float load_as_f32(const T* p);
template <> __device__ __forceinline__ float load_as_f32<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_as_f32<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }

template <typename T> __device__ __forceinline__ void store_from_f32(T* p, float v);
template <> __device__ __forceinline__ void store_from_f32<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void store_from_f32<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }

// Four consecutive elements at once (the address must be a multiple of four elements).
template <typename T> __device__ __forceinline__ f32x4 load4_as_f32(const T* p);
template <> __device__ __forceinline__ f32x4 load4_as_f32<float>(const float* p) { return *(const f32x4*)p; }
template <> __device__ __forceinline__ f32x4 load4_as_f32<uint16_t>(const uint16_t* p) {
  const uint2 u = *(const uint2*)p;
  f32x4 v;
  v[0] = __uint_as_float(u.x << 16);
  v[1] = __uint_as_float(u.x & 0xffff0000u);
  v[2] = __uint_as_float(u.y << 16);
  v[3] = __uint_as_float(u.y & 0xffff0000u);
  return v;
}
template <typename T> __device__ __forceinline__ void store4_from_f32(T* p, const f32x4& v);
template <> __device__ __forceinline__ void store4_from_f32<float>(float* p, const f32x4& v) { *(f32x4*)p = v; }
template <> __device__ __forceinline__ void store4_from_f32<uint16_t>(uint16_t* p, const f32x4& v) {
  uint2 u;
  u.x = (unsigned)f32_to_bf16(v[0]) | ((unsigned)f32_to_bf16(v[1]) << 16);
  u.y = (unsigned)f32_to_bf16(v[2]) | ((unsigned)f32_to_bf16(v[3]) << 16);
  *(uint2*)p = u;
}

// Workgroup id -> (row tile mb, column tile ct).  Workgroups are dealt round-robin
// to the 8 XCDs, each with its own L2, so id g runs on XCD g%8 as that XCD's
// (g/8)-th workgroup.
//
// "Contiguous" map, for passes whose tiles all cost the same: tiles are put in a
// line -- column tiles in groups of 8, all MB row tiles of a group together, so
// that neighbours in the line share both operand panels -- and the line is cut
// into 8 equal pieces, one per XCD.  Every XCD gets the same number of tiles
// (+-1) and the tiles resident together on it are neighbours in the line.
__device__ __forceinline__ void tile_from_line(int L, int MB, int CT, int& mb, int& ct) {
  const int full = 8 * MB;                 // tiles in a full group
  const int grp = L / full;
  const int rem = L - grp * full;
  const int gs = min(8, CT - 8 * grp);     // column tiles in this group (last may be ragged)
  mb = rem / gs;
  ct = 8 * grp + (rem - mb * gs);
}
// Workgroup g of a grid of grid_contiguous(n) -> position in the line, for the first n tiles.
__device__ __forceinline__ bool line_contiguous(int g, int n, int& L) {
  const int per = (n + 7) >> 3;
  const int s = g >> 3;
  L = (g & 7) * per + s;
  return s < per && L < n;
}
__host__ __device__ static inline int grid_contiguous(int n) { return 8 * ((n + 7) / 8); }

// Tail plan for the equal-cost passes.  With S workgroup slots on the chip (two per CU)
// and T tiles, the first nFull = S*floor(T/S) tiles are computed whole, one workgroup
// each, in full rounds.  The remaining nTail tiles would occupy only part of the chip for
// a whole tile time; instead their nTail*nch reduction chunks are dealt out in equal runs
// of `units` consecutive chunks to nTailWg workgroups (a run covers at most two tiles).
// Each run writes its accumulators to a scratch slot and a fix-up kernel adds the slots
// of a tile in run order, so the result does not depend on timing.
struct TailPlan {
  int nFull, nTail, units, nTailWg;
};
constexpr int TAIL_SLOT_FLOATS = 64 * NT;   // one wavefront-layout accumulator image (64 KB)

// "Dealt" map, for the input-gradient pass whose column tiles are sorted by
// decreasing cost: column tile ct goes to XCD ct%8 (so every XCD gets the same mix
// of heavy and light tiles and starts with its heaviest), and the MB row tiles
// that share its operand panel follow each other on that XCD.
__device__ __forceinline__ bool tile_dealt(int g, int MB, int CT, int& mb, int& ct) {
  const int s = g >> 3;
  const int lc = s / MB;
  mb = s - lc * MB;
  ct = lc * 8 + (g & 7);
  return ct < CT;
}
static inline int grid_dealt(int MB, int CT) { return 8 * ((CT + 7) / 8) * MB; }

// ---------------------------------------------------------------------------
// Staging.  Operand tiles go from global memory straight into LDS with the
// gfx950 16-byte LDS-DMA load (global_load_lds_dwordx4): no staging registers,
// no LDS store instructions.  One such instruction moves 64 x 16 bytes; lane l's
// 16 bytes land at (wave-uniform LDS base) + 16*l, while each lane chooses its
// own global address.  The LDS image of a tile is therefore fixed by lane order,
// and a tile (128 x 32 floats = 1024 slots of 16 bytes) takes 16 wave-level
// instructions: wavefront wv issues number i = 0..3 into slots
// [(4*wv+i)*64, +64).  Two tile images are used:
//
//   row image  [kk][128]: reduction index kk is the row, 32 slots per row.
//              slot = kk*32 + cq  ->  lane l of (wv,i) fetches row 8*wv+2*i+l/32,
//              float columns 4*(l%32)..+3.  MFMA operands are read with 4-byte
//              LDS reads along a row (conflict free).
//   col image  [m][8 slots], XOR-swizzled: tile row m holds its 32 reduction
//              elements as 8 slots, logical slot kq stored at position kq^(m&7).
//              Lane l of (wv,i) fetches row 32*wv+8*i+l/8, logical slot
//              (l%8)^(l/8).  MFMA operands are read with one 16-byte LDS read per
//              four reduction steps; the swizzle makes 8 consecutive rows hit 8
//              different 16-byte bank groups.
//
// Lanes whose element must be zero (padding tap, reduction tail, column block
// past the end) fetch from a small zero-filled page instead.
// ---------------------------------------------------------------------------
#define CS_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define CS_LPTR(p) ((__attribute__((address_space(3))) void*)(p))
// Tables a kernel only reads and whose address is wave-uniform: loads through a pointer
// to the constant address space are scalar loads.
#define CS_CONST __attribute__((address_space(4)))

// A pointer the compiler must treat as an opaque wave-uniform value (no folding of the
// arithmetic that produced it into later address computations).
__device__ __forceinline__ const char* opaque_uniform(const void* p) {
  const unsigned long long v = (unsigned long long)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (const char*)(((unsigned long long)hi << 32) | lo);
}

// The same load with the address split into a wave-uniform base and a 32-bit per-lane byte
// offset.  The instruction then takes the base from scalar registers and the lane offset as
// it is, so an operand whose lanes keep their offsets from chunk to chunk costs no vector
// ALU work at all: only the scalar base moves.  (The empty asm keeps the zero-extension of
// the offset next to the addition, which is the form the instruction selector recognises.)
__device__ __forceinline__ void dma16_uv(const char* base_uniform, unsigned& lane_off, float* lds_uniform) {
  asm volatile("" : "+v"(lane_off));
  __builtin_amdgcn_global_load_lds(CS_GPTR(base_uniform + lane_off), CS_LPTR(lds_uniform), 16, 0, 0);
}

// Reduction order inside a chunk.  MFMA step ks = 4*j + t (j, t in 0..3) multiplies
// the element pair kk = 8*j + t (lanes 0..31) and kk = 8*j + 4 + t (lanes 32..63),
// which is what a 16-byte read of col-image slot 2*j + lane/32 delivers.
// Col image: tile row m keeps its eight 16-byte slots (four reduction steps each) in the
// order slot = kq ^ col_key(m).  The key is chosen by measurement: with (m >> 1) & 7 a
// wavefront's 16-byte LDS reads run at 256 bytes per clock, with m & 7 at half of that.
__device__ __forceinline__ int col_key(int row) { return (row >> 1) & 7; }

// Tile shapes of the fp32 kernels, by the template parameter MI:
//   MI = 2: 128 rows, MI = 1: 64 rows -- four wavefronts as 2 x 2, each MI x 2 accumulator blocks;
//   MI = 3:  96 rows -- four wavefronts side by side (1 x 4), each 3 x 1 blocks: every wavefront does the
//            same work, which a 2 x 2 arrangement of three row blocks could not give.
//   MI = 4: 128 rows x 96 columns -- four wavefronts on top of each other (4 x 1), each 1 x 3 blocks: for passes
//            whose column extent is at most 96 (the weight gradient of a layer with C*R*S <= 96), where the fourth
//            column block of the other shapes would multiply padding.
// The other shapes are 128 columns wide.  RB = 32-row blocks per wavefront, NJ = 32-column blocks per wavefront.
template <int MI>
struct Shape {
  static_assert(MI >= 1 && MI <= 4, "tile shapes: 64, 128 or 96 rows, or 128 rows x 96 columns");
  static constexpr int RB = MI == 4 ? 1 : MI;                      // row blocks per wavefront
  static constexpr int NJ = MI == 3 ? 1 : MI == 4 ? 3 : 2;         // column blocks per wavefront
  static constexpr int ROWS = MI == 3 ? 96 : MI == 4 ? 128 : 64 * MI;  // tile rows
  static constexpr int NLOAD = ROWS / 32;              // A-operand DMA loads per wavefront and chunk
  static constexpr int WROWS = ROWS / 4;               // A rows a wavefront stages
  __device__ static __forceinline__ int row0(int wave) { return MI == 3 ? 0 : MI == 4 ? wave * 32 : (wave >> 1) * (32 * MI); }
  __device__ static __forceinline__ int col0(int wave) { return MI == 3 ? wave * 32 : MI == 4 ? 0 : (wave & 1) * 64; }
  __device__ static __forceinline__ int colblk0(int wave) { return MI == 3 ? wave : MI == 4 ? 0 : (wave & 1) * 2; }
};

template <int NBLK>
struct FragN {         // operands of four MFMA steps (one j) for NBLK of the wavefront's 32-wide blocks
  f32x4 v[NBLK];       // v[blk][t]
};
using Frag = FragN<2>;

template <bool COL, int NBLK>
__device__ __forceinline__ void read_frag(FragN<NBLK>& f, const float* tile, int wbase, int lane, int j, int blk1) {
  if constexpr (COL) {
    const int u = col_key(lane & 31), h = lane >> 5;
    const int slot = (wbase + (lane & 31)) * 8 + ((2 * j + h) ^ u);
#pragma unroll
    for (int b = 0; b < NBLK; ++b) f.v[b] = *(const f32x4*)(tile + slot * 4 + b * (32 * 8 * 4));
  } else {
    static_assert(NBLK <= 3, "row images feed up to three blocks");
    // The second block lies blk1 = 32 floats to the right.  blk1 is an opaque register (see
    // opaque_block_offset), so the two blocks keep separate base registers and the reads of
    // rows t, t+1 of one block (512 bytes apart) pair up into LDS reads with 256-byte offset
    // units, which reach every j and t from that one base.
    const float* p = tile + (8 * j + 4 * (lane >> 5)) * BM + wbase + (lane & 31);
#pragma unroll
    for (int t = 0; t < 4; ++t) f.v[0][t] = p[t * BM];
    if constexpr (NBLK >= 2) {
      const float* q = p + blk1;
#pragma unroll
      for (int t = 0; t < 4; ++t) f.v[1][t] = q[t * BM];
    }
    if constexpr (NBLK == 3) {
      const float* q2 = p + 2 * blk1;
#pragma unroll
      for (int t = 0; t < 4; ++t) f.v[2][t] = q2[t * BM];
    }
  }
}

__device__ __forceinline__ int opaque_block_offset() {
  int o = 32;
  asm volatile("" : "+v"(o));
  return o;
}

// Four reduction steps on the wavefront's MI x NJ accumulator blocks (sixteen MFMAs for MI = 2, twelve for MI = 3).
template <int MI>
__device__ __forceinline__ void mfma_group(const FragN<Shape<MI>::RB>& a, const FragN<Shape<MI>::NJ>& b,
                                           f32x16 (&acc)[Shape<MI>::RB][Shape<MI>::NJ]) {
#pragma unroll
  for (int t = 0; t < 4; ++t) {
#pragma unroll
    for (int i = 0; i < Shape<MI>::RB; ++i) {
#pragma unroll
      for (int j = 0; j < Shape<MI>::NJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[i][t], b.v[j][t], acc[i][j], 0, 0, 0);
    }
  }
}

// Scheduling fence: LDS reads and MFMAs keep their order across it, while vector/scalar
// ALU and memory instructions (the next chunk's address arithmetic and DMA issue) may
// move, so that they issue in the shadow of the MFMAs instead of in front of them.
#define CS_FENCE() __builtin_amdgcn_sched_barrier(0x0002 | 0x0004 | 0x0010)

// Main loop shared by the three passes.  A loader stages one operand; per chunk it is
// driven as begin(ch, live), issue(0..3, dst), end(): issue(i, dst) starts LDS-DMA load
// number i of this wavefront's share of chunk ch into the wave-uniform LDS address dst
// (chunks are requested in increasing order, once each; live = false marks chunks past the
// last one, whose loads must stay harmless so that the loop body needs no branch).  LDS
// holds [A stage0][A stage1][B stage0][B stage1].
// The A operand has Shape<LA::MI>::ROWS rows (128, 64 for a short last row tile, or 96), i.e. ROWS / 32 loads per
// wavefront and chunk.
template <class LA, class LB>
__device__ __forceinline__ void issue_all(LA& la, LB& lb, int ch, float* ta, float* tb, int wv, bool live) {
  constexpr int NLOAD = Shape<LA::MI>::NLOAD;
  la.begin(ch, live);
  lb.begin(ch, live);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i < NLOAD) la.issue(i, ta + (wv * NLOAD + i) * 256);
    lb.issue(i, tb + (wv * 4 + i) * 256);
  }
  la.end();
  lb.end();
}


// One barrier per chunk: after the barrier that publishes chunk ch, a wavefront issues the
// DMA loads of chunk ch+1 (they have one chunk time to land), runs G2,G3 of chunk ch-1
// from registers while the LDS reads of G0,G1 of chunk ch are in flight, then G0,G1 of
// chunk ch while G2,G3 are being read.
template <class LA, class LB>
__device__ __forceinline__ void gemm_mainloop(LA& la, LB& lb, int ch_begin, int ch_end, float* smem,
                                              f32x16 (&acc)[Shape<LA::MI>::RB][Shape<LA::MI>::NJ]) {
  constexpr bool AC = LA::COL, BC = LB::COL;
  constexpr int MI = LA::MI;
  static_assert(MI == 2 || AC, "the 64- and 96-row tiles need a col-image A operand");
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wa = Shape<MI>::row0(wv), wb = Shape<MI>::col0(wv);
  if (ch_begin >= ch_end) return;
  const int blk1 = opaque_block_offset();
  FragN<Shape<MI>::RB> a0, a1;
  FragN<Shape<MI>::NJ> b0, b1;
  // prologue: chunk ch_begin into stage 0
  issue_all(la, lb, ch_begin, smem, smem + 2 * TILE_F, wv, true);
  __syncthreads();  // includes the wait for this wavefront's own DMA loads
  read_frag<AC>(a0, smem, wa, lane, 0, blk1);
  read_frag<BC>(b0, smem + 2 * TILE_F, wb, lane, 0, blk1);
  read_frag<AC>(a1, smem, wa, lane, 1, blk1);
  read_frag<BC>(b1, smem + 2 * TILE_F, wb, lane, 1, blk1);
  issue_all(la, lb, ch_begin + 1, smem + TILE_F, smem + 3 * TILE_F, wv, ch_begin + 1 < ch_end);
  CS_FENCE();
  mfma_group<MI>(a0, b0, acc);
  CS_FENCE();
  read_frag<AC>(a0, smem, wa, lane, 2, blk1);
  read_frag<BC>(b0, smem + 2 * TILE_F, wb, lane, 2, blk1);
  CS_FENCE();
  mfma_group<MI>(a1, b1, acc);
  CS_FENCE();
  read_frag<AC>(a1, smem, wa, lane, 3, blk1);
  read_frag<BC>(b1, smem + 2 * TILE_F, wb, lane, 3, blk1);
  __syncthreads();
  int cur = TILE_F;  // float offset of the stage that holds chunk ch: TILE_F or 0
  for (int ch = ch_begin + 1; ch < ch_end; ++ch) {
    const float* As = smem + cur;
    const float* Bs = smem + 2 * TILE_F + cur;
    issue_all(la, lb, ch + 1, smem + (cur ^ TILE_F), smem + 2 * TILE_F + (cur ^ TILE_F), wv, ch + 1 < ch_end);
    CS_FENCE();
    mfma_group<MI>(a0, b0, acc);  // G2 of chunk ch-1
    CS_FENCE();
    read_frag<AC>(a0, As, wa, lane, 0, blk1);
    read_frag<BC>(b0, Bs, wb, lane, 0, blk1);
    CS_FENCE();
    mfma_group<MI>(a1, b1, acc);  // G3 of chunk ch-1
    CS_FENCE();
    read_frag<AC>(a1, As, wa, lane, 1, blk1);
    read_frag<BC>(b1, Bs, wb, lane, 1, blk1);
    CS_FENCE();
    mfma_group<MI>(a0, b0, acc);  // G0 of chunk ch
    CS_FENCE();
    read_frag<AC>(a0, As, wa, lane, 2, blk1);
    read_frag<BC>(b0, Bs, wb, lane, 2, blk1);
    CS_FENCE();
    mfma_group<MI>(a1, b1, acc);  // G1 of chunk ch
    CS_FENCE();
    read_frag<AC>(a1, As, wa, lane, 3, blk1);
    read_frag<BC>(b1, Bs, wb, lane, 3, blk1);
    __syncthreads();
    cur ^= TILE_F;
  }
  mfma_group<MI>(a0, b0, acc);  // G2, G3 of the last chunk
  mfma_group<MI>(a1, b1, acc);
}

// Four reduction steps that start a tile: the first step writes the accumulators (C operand zero) instead of
// adding to them, so a new tile needs no clearing pass over the accumulator registers.
template <int MI>
__device__ __forceinline__ void mfma_group_first(const FragN<MI>& a, const FragN<Shape<MI>::NJ>& b,
                                                 f32x16 (&acc)[MI][Shape<MI>::NJ]) {
  constexpr int NJ = Shape<MI>::NJ;
  f32x16 zero;
#pragma unroll
  for (int v = 0; v < 16; ++v) zero[v] = 0.f;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[i][0], b.v[j][0], zero, 0, 0, 0);
#pragma unroll
  for (int t = 1; t < 4; ++t) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[i][t], b.v[j][t], acc[i][j], 0, 0, 0);
  }
}

// The same loop over a stream of tiles that all have nch chunks: a workgroup computes its tiles one after the
// other and the chunk pipeline runs on across tile boundaries -- the first loads of the next tile are issued
// while the last chunk of the current one is multiplied, and a finished tile's accumulators are stored between
// two MFMA groups of the next tile's first chunk.  For tiles with short reductions (a few chunks) this keeps
// the per-tile prologue, epilogue and workgroup launch off the critical path.
// `tiles` supplies the stream: advance() moves on to the next tile to load (false: none left), make_a() builds
// the A loader of that tile; its B loader is built by make_b(), or, when same_b() says that the tile has the
// column tile of the one before, the current B loader is only restarted (restart()); store(acc) stores the
// oldest tile not yet stored (tiles are stored in the order they were loaded).
// lastg = groups of eight reduction elements that hold data in a tile's last chunk (1..4): the third and fourth
// group of that chunk are skipped when they are all padding (their A operand is zero).
template <class LA, class LB, class Tiles>
__device__ __forceinline__ void gemm_stream(Tiles& tiles, int nch, float* smem, int lastg = 4) {
  constexpr bool AC = LA::COL, BC = LB::COL;
  constexpr int MI = LA::MI;
  static_assert(MI == 2 || AC, "the 64- and 96-row tiles need a col-image A operand");
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wa = Shape<MI>::row0(wv), wb = Shape<MI>::col0(wv);
  if (!tiles.advance()) return;
  LA la = tiles.make_a();
  LB lb = tiles.make_b();
  const int blk1 = opaque_block_offset();
  f32x16 acc[MI][Shape<MI>::NJ];
  // Issues the loads of the chunk that follows chunk ch of the tile being loaded; false at the end of the stream.
  auto issue_next = [&](int ch, float* ta, float* tb) -> bool {
    if (ch + 1 < nch) {
      issue_all(la, lb, ch + 1, ta, tb, wv, true);
      return true;
    }
    if (!tiles.advance()) return false;
    la = tiles.make_a();
    if (tiles.same_b()) lb.restart();
    else lb = tiles.make_b();
    issue_all(la, lb, 0, ta, tb, wv, true);
    return true;
  };
  FragN<MI> a0, a1;
  FragN<Shape<MI>::NJ> b0, b1;
  issue_all(la, lb, 0, smem, smem + 2 * TILE_F, wv, true);
  __syncthreads();
  read_frag<AC>(a0, smem, wa, lane, 0, blk1);
  read_frag<BC>(b0, smem + 2 * TILE_F, wb, lane, 0, blk1);
  read_frag<AC>(a1, smem, wa, lane, 1, blk1);
  read_frag<BC>(b1, smem + 2 * TILE_F, wb, lane, 1, blk1);
  int ch = 0;   // chunk, within its tile, whose fragments are in registers
  bool more = issue_next(ch, smem + TILE_F, smem + 3 * TILE_F);
  CS_FENCE();
  mfma_group_first(a0, b0, acc);
  CS_FENCE();
  read_frag<AC>(a0, smem, wa, lane, 2, blk1);
  read_frag<BC>(b0, smem + 2 * TILE_F, wb, lane, 2, blk1);
  CS_FENCE();
  mfma_group<MI>(a1, b1, acc);
  CS_FENCE();
  read_frag<AC>(a1, smem, wa, lane, 3, blk1);
  read_frag<BC>(b1, smem + 2 * TILE_F, wb, lane, 3, blk1);
  __syncthreads();
  int cur = TILE_F;
  while (more) {
    ++ch;
    const bool newtile = ch == nch;   // the chunk entered now is the first of the next tile
    ch = newtile ? 0 : ch;
    const float* As = smem + cur;
    const float* Bs = smem + 2 * TILE_F + cur;
    float* ta = smem + (cur ^ TILE_F);
    float* tb = smem + 2 * TILE_F + (cur ^ TILE_F);
    // The chunk to load now: the next one of this tile, or the first one of the next tile (loaders rebuilt;
    // register work only, so that the loads themselves sit in the straight-line code below, among the MFMAs).
    // At the end of the stream the loads are issued once more as harmless dummies (live = false).
    int chn = ch + 1;
    bool live = true;
    if (chn == nch) {
      chn = 0;
      live = tiles.advance();
      if (live) {
        la = tiles.make_a();
        if (tiles.same_b()) lb.restart();
        else lb = tiles.make_b();
      }
    }
    if (!newtile) {
      issue_all(la, lb, chn, ta, tb, wv, live);
      CS_FENCE();
      mfma_group<MI>(a0, b0, acc);  // G2 of the chunk before
      CS_FENCE();
      read_frag<AC>(a0, As, wa, lane, 0, blk1);
      read_frag<BC>(b0, Bs, wb, lane, 0, blk1);
      CS_FENCE();
      mfma_group<MI>(a1, b1, acc);  // G3 of the chunk before
      CS_FENCE();
      read_frag<AC>(a1, As, wa, lane, 1, blk1);
      read_frag<BC>(b1, Bs, wb, lane, 1, blk1);
      CS_FENCE();
      mfma_group<MI>(a0, b0, acc);  // G0 of this chunk
    } else {
      issue_all(la, lb, chn, ta, tb, wv, live);
      CS_FENCE();
      if (lastg > 2) mfma_group<MI>(a0, b0, acc);  // G2 of the chunk before, the last of its tile
      CS_FENCE();
      read_frag<AC>(a0, As, wa, lane, 0, blk1);
      read_frag<BC>(b0, Bs, wb, lane, 0, blk1);
      CS_FENCE();
      if (lastg > 3) mfma_group<MI>(a1, b1, acc);  // G3 of the chunk before
      CS_FENCE();
      read_frag<AC>(a1, As, wa, lane, 1, blk1);
      read_frag<BC>(b1, Bs, wb, lane, 1, blk1);
      CS_FENCE();
      tiles.store(acc);
      mfma_group_first(a0, b0, acc);  // G0 of this chunk, starting a tile
    }
    CS_FENCE();
    read_frag<AC>(a0, As, wa, lane, 2, blk1);
    read_frag<BC>(b0, Bs, wb, lane, 2, blk1);
    CS_FENCE();
    mfma_group<MI>(a1, b1, acc);  // G1 of this chunk
    CS_FENCE();
    read_frag<AC>(a1, As, wa, lane, 3, blk1);
    read_frag<BC>(b1, Bs, wb, lane, 3, blk1);
    __syncthreads();
    cur ^= TILE_F;
    more = live;
  }
  if (lastg > 2) mfma_group<MI>(a0, b0, acc);  // G2, G3 of the last chunk
  if (lastg > 3) mfma_group<MI>(a1, b1, acc);
  tiles.store(acc);
}

// A workgroup's contiguous run [begin, end) of a line of T equal tiles, for a grid of W persistent workgroups
// (W a multiple of 8).  Workgroups are dealt to the XCDs in contiguous blocks, so the runs resident together on
// one XCD are neighbours in the line.
__device__ __forceinline__ void stream_run(int T, int& begin, int& end) {
  const int W = gridDim.x;
  const int w = (blockIdx.x & 7) * (W >> 3) + (blockIdx.x >> 3);
  begin = (int)((int64_t)T * w / W);
  end = (int)((int64_t)T * (w + 1) / W);
}

// Position of accumulator register v of a 32x32 MFMA block inside the block.
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

}  // namespace cs
