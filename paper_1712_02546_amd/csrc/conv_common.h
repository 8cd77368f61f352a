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

namespace cs {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int NT = 256;             // threads per workgroup: 4 wavefronts in a 2x2 grid
constexpr int BM = 128;             // tile rows  (GEMM M)
constexpr int BN = 128;             // tile cols  (GEMM N) = 4 column blocks of 32
constexpr int BK = 32;              // reduction elements per staged chunk
constexpr int LDT = 129;            // LDS row pitch for operands stored transposed (scalar stores)
constexpr int LDV = 132;            // LDS row pitch for operands stored as float4 rows
constexpr int STAGE = BK * LDV;     // floats per operand per buffer
constexpr int SMEM_BYTES = 4 * STAGE * 4;  // A and B, double buffered

struct Geo {
  int N, Np, NB;                    // batch, padded batch, Np/32
  int C, H, W, K, R, S, P, Q;
  int sh, sw, ph, pw;
  int k0, Ks;
  int HW, PQ, RS, CRS;
};

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

// Workgroup id -> (row tile mb, column tile ct).  Workgroups are dealt round-robin
// to the 8 XCDs, each with its own L2, so id g runs on XCD g%8 as that XCD's
// (g/8)-th workgroup.
//
// "Contiguous" map, for passes whose tiles all cost the same: tiles are put in a
// line -- column tiles in groups of 8, all MB row tiles of a group together, so
// that neighbours in the line share both operand panels -- and the line is cut
// into 8 equal pieces, one per XCD.  Every XCD gets the same number of tiles
// (+-1) and the tiles resident together on it are neighbours in the line.
__device__ __forceinline__ bool tile_contiguous(int g, int MB, int CT, int& mb, int& ct) {
  const int T = MB * CT;
  const int per = (T + 7) >> 3;
  const int s = g >> 3;
  const int L = (g & 7) * per + s;
  if (s >= per || L >= T) return false;
  const int full = 8 * MB;                 // tiles in a full group
  const int grp = L / full;
  const int rem = L - grp * full;
  const int gs = min(8, CT - 8 * grp);     // column tiles in this group (last may be ragged)
  mb = rem / gs;
  ct = 8 * grp + (rem - mb * gs);
  return true;
}
static inline int grid_contiguous(int MB, int CT) { return 8 * ((MB * CT + 7) / 8); }

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

__device__ __forceinline__ f32x4 masked(const f32x4& v, bool ok) {
  f32x4 o;
  o.x = ok ? v.x : 0.f;
  o.y = ok ? v.y : 0.f;
  o.z = ok ? v.z : 0.f;
  o.w = ok ? v.w : 0.f;
  return o;
}

// One staged chunk: 16 reduction steps of four 32x32x2 fp32 MFMAs per wavefront.
// As/Bs are [BK][lda]/[BK][ldb] with the reduction index as the row.  In
// v_mfma_f32_32x32x2_f32 lane l supplies A[row l%32][k l/32] and B[k l/32][col l%32].
__device__ __forceinline__ void mfma_chunk(const float* __restrict__ As, int lda,
                                           const float* __restrict__ Bs, int ldb,
                                           int wm, int wn, int lane, f32x16 (&acc)[2][2]) {
  const float* ap = As + (lane >> 5) * lda + wm * 64 + (lane & 31);
  const float* bp = Bs + (lane >> 5) * ldb + wn * 64 + (lane & 31);
  // Operands of step ks+1 are read from LDS before the MFMAs of step ks are issued.
  float a0 = ap[0], a1 = ap[32], b0 = bp[0], b1 = bp[32];
#pragma unroll
  for (int ks = 0; ks < BK / 2; ++ks) {
    float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
    if (ks + 1 < BK / 2) {
      na0 = ap[2 * (ks + 1) * lda];
      na1 = ap[2 * (ks + 1) * lda + 32];
      nb0 = bp[2 * (ks + 1) * ldb];
      nb1 = bp[2 * (ks + 1) * ldb + 32];
    }
    __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the MFMAs they overlap with
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
  }
}

// Software-pipelined main loop shared by the three passes.  A loader stages one
// operand: load(ch) issues the global reads of chunk ch into registers (chunks
// are requested in increasing order, once each), store(buf) writes them to LDS.
template <class LA, class LB>
__device__ __forceinline__ void gemm_mainloop(LA& la, LB& lb, int ch_begin, int ch_end,
                                              float* smem, f32x16 (&acc)[2][2]) {
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // LDS map: [A buf0][A buf1][B buf0][B buf1]; offsets (not pointers) select the
  // buffer so that every access stays a plain LDS instruction.
  if (ch_begin >= ch_end) return;
  la.load(ch_begin);
  lb.load(ch_begin);
  la.store(smem);
  lb.store(smem + 2 * STAGE);
  __syncthreads();
  int cur = 0;
#ifndef CS_EXP
#define CS_EXP 0
#endif
  for (int ch = ch_begin; ch < ch_end; ++ch) {
    const bool more = ch + 1 < ch_end;
    if (more && !(CS_EXP & 1)) {
      la.load(ch + 1);
      lb.load(ch + 1);
    }
    if (!(CS_EXP & 4)) mfma_chunk(smem + cur, LA::LD, smem + 2 * STAGE + cur, LB::LD, wm, wn, lane, acc);
    cur ^= STAGE;
    if (more && !(CS_EXP & 1)) {
      la.store(smem + cur);
      lb.store(smem + 2 * STAGE + cur);
    }
    if (!(CS_EXP & 2)) __syncthreads();
  }
}

// Position of accumulator register v of a 32x32 MFMA block inside the block.
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

}  // namespace cs
