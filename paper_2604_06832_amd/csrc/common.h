// Shared device-side types and helpers for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bd {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned short u16;

constexpr int kWave = 64;
constexpr int kWGThreads = 256;          // every kernel here runs 4 wavefronts per workgroup
constexpr int kWavesPerWG = 4;

// ---- operand layouts -----------------------------------------------------------------------------
// All matrix operands live in HBM in the order the 16x16x32 bf16 MFMA consumes them, so that one
// wavefront's operand load is one contiguous, 16-byte-per-lane, 1 KiB read.
//
//  A/B fragment of a [16 rows] x [32 k] tile: lane l holds row (l & 15), k = 8*(l >> 4) .. +7.
//  C/D fragment of a [16 x 16] tile (4 fp32 per lane): lane l holds column (l & 15),
//  rows 4*(l >> 4) .. +3.
//
//  Packed weight  W[N][K] (N % 16 == 0):  tile (nt, ks) at ((nt*KS + ks)*64 + lane)*8 + e
//       = W[nt*16 + (lane & 15)][ks*32 + 8*(lane >> 4) + e],   KS = ceil(K/32), zero beyond K.
//  Packed activation X[M][K] (MT = ceil(M/16)): tile (ks, mt) at ((ks*MT + mt)*64 + lane)*8 + e
//       = X[mt*16 + (lane & 15)][ks*32 + 8*(lane >> 4) + e].
__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

__device__ inline u16 f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);     // round to nearest even (inputs here are finite)
  return (u16)(u >> 16);
}
__device__ inline float bf16_bits_to_f32(u16 b) { return __uint_as_float(((uint32_t)b) << 16); }

// Index of element (m, k) inside a packed activation with MT row tiles.
__device__ inline size_t xp_index(int m, int k, int MT) {
  int ks = k >> 5, kq = (k >> 3) & 3, e = k & 7;
  int mt = m >> 4, lane = kq * 16 + (m & 15);
  return (((size_t)ks * MT + mt) * 64 + lane) * 8 + e;
}

// In-block visibility of the block's key jb (0-based index inside the block) for the block's query row `row`
// (Sec. 3.3 mask rules; Alg. 1 draft / verify masks; Alg. 2 quadratic mask).  mode 0: all visible; 1: causal;
// 2 + (B << 8): B groups of B+1 rows, a group's first row sees the first rows of the groups up to its own, every other
// row sees the rows of its own group.  (Keys of the committed prefix are visible to every row.)
// QUAD is a compile-time switch: the kernels of ordinary forwards are built without the quadratic rule (its index
// arithmetic costs registers in every phase of the persistent kernels), the quadratic step runs its own instantiations.
template <bool QUAD>
__device__ inline bool block_key_visible(int mode, int row, int jb) {
  if constexpr (!QUAD) {
    return mode == 0 || jb <= row;
  } else {
    const int W = (mode >> 8) + 1;
    const int gi = row / W, gj = row - gi * W, ki = jb / W, kj = jb - ki * W;
    return gj == 0 ? (kj == 0 && ki <= gi) : ki == gi;
  }
}

// State that lives on the device so that replayed launch sequences need no new kernel arguments.
struct DevState {
  int n;             // committed context length
  int seeded;        // 1 if the current denoise call revealed position 0 from the carry
  int carry_cand;    // prediction for position n
  float carry_conf;
  int error;         // sticky device-side error flag (bounded waits)
  int skip;          // bd_decode_block: the current block has no masked position left; its remaining steps do nothing
  int steps;         // bd_decode_block: denoising forwards that really ran for the current block
};

}  // namespace bd
