// bf16 MFMA main loop shared by the projection GEMMs and the LM-head kernel.
//
//   C[M,N] = X[M,K] * W[N,K]^T      X = activations, W = weights, both K-contiguous (row-major).
//
// Design for the verify step's shapes (M = 20..4352 packed query rows, weights far larger than
// activations): a workgroup of 4 waves owns BM = 32*MT rows and 4*NT*32 weight rows; the four
// waves sit side by side along N.
//   * Weights stream HBM -> VGPR directly, never through LDS: every weight element is needed by
//     exactly one wave.  Lane (n, g) of a wave reads 64 contiguous bytes of weight row n per
//     64-wide K tile (k = 32g .. 32g+31), i.e. two lanes cover one full 128-byte line.
//   * Activations go through LDS (shared by the 4 waves), stored in MFMA fragment order so that
//     every fragment read is one conflict-free 1 KiB ds_read_b128 sweep.
//   * The contraction index inside a K tile is permuted (MFMA step s of lane group g multiplies
//     k = 32g + 8s + j); sums do not depend on the order of k, and both operands use the same
//     permutation, so no data movement is needed to make the weight loads contiguous.
//   * SWAP = true issues mfma(W, X) instead of mfma(X, W): the accumulator then holds C^T tiles
//     (rows = weight rows, lane = token), which makes per-token reductions over N in-lane.
#pragma once
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;   // K tile (elements)

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Accumulator element i of lane `lane` in a 32x32 MFMA tile: row, col inside the tile.
__device__ __forceinline__ int acc_row(int lane, int i) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }
__device__ __forceinline__ int acc_col(int lane) { return lane & 31; }

template <int MT, int NT, bool SWAP>
struct MfmaGemm {
  static constexpr int BM = 32 * MT;
  static constexpr int LDS_STAGE_BYTES = MT * 4 * 1024;        // MT row tiles x 4 K-steps x 1 KiB
  static constexpr int LDS_BYTES = 2 * LDS_STAGE_BYTES;

  // x_rows[i]: global pointer to the start of this thread's i-th 16-byte activation chunk at k=0
  //            (already includes the row and the (g, s) offset inside a K tile), i < MT.
  // x_lds[i]:  byte offset of that chunk inside an LDS stage.
  // w_rows[ni]: pointer to weight row (k = 32*g) for N tile ni of this lane.
  // nk: number of K tiles.
  __device__ static __forceinline__ void run(f32x16 (&acc)[MT][NT], const bf16* const (&x_rows)[MT],
                                             const int (&x_lds)[MT], const bf16* const (&w_rows)[NT], int nk,
                                             char* lds) {
    const int lane = threadIdx.x & 63;
    u32x4 xreg[MT];
    u32x4 wnext[NT][4];
#pragma unroll
    for (int i = 0; i < MT; ++i) xreg[i] = *(const u32x4*)(x_rows[i]);
#pragma unroll
    for (int ni = 0; ni < NT; ++ni)
#pragma unroll
      for (int s = 0; s < 4; ++s) wnext[ni][s] = *(const u32x4*)(w_rows[ni] + s * 8);
#pragma unroll
    for (int i = 0; i < MT; ++i) *(u32x4*)(lds + x_lds[i]) = xreg[i];
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      u32x4 wcur[NT][4];
#pragma unroll
      for (int ni = 0; ni < NT; ++ni)
#pragma unroll
        for (int s = 0; s < 4; ++s) wcur[ni][s] = wnext[ni][s];
      const bool more = kt + 1 < nk;
      if (more) {
        const int koff = (kt + 1) * kBK;
#pragma unroll
        for (int i = 0; i < MT; ++i) xreg[i] = *(const u32x4*)(x_rows[i] + koff);
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
#pragma unroll
          for (int s = 0; s < 4; ++s) wnext[ni][s] = *(const u32x4*)(w_rows[ni] + koff + s * 8);
      }
      const char* stage = lds + (kt & 1) * LDS_STAGE_BYTES;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int mi = 0; mi < MT; ++mi) {
          bf16x8 xf = as_bf16x8(*(const u32x4*)(stage + ((mi * 4 + s) * 64 + lane) * 16));
#pragma unroll
          for (int ni = 0; ni < NT; ++ni) {
            bf16x8 wf = as_bf16x8(wcur[ni][s]);
            if (SWAP) acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[mi][ni], 0, 0, 0);
            else      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, wf, acc[mi][ni], 0, 0, 0);
          }
        }
      }
      if (more) {
        char* nstage = lds + ((kt + 1) & 1) * LDS_STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < MT; ++i) *(u32x4*)(nstage + x_lds[i]) = xreg[i];
      }
      __syncthreads();
    }
  }

  // Chunk assignment of thread t for the activation tile: chunk q = i*256 + t covers
  // (row, g, s) with g = q / (BM*4), row = (q % (BM*4)) / 4, s = q % 4.
  __device__ static __forceinline__ void chunk_of(int i, int& row, int& g, int& s) {
    int q = i * 256 + threadIdx.x;
    g = q / (BM * 4);
    int rem = q % (BM * 4);
    row = rem >> 2;
    s = rem & 3;
  }
  __device__ static __forceinline__ int chunk_lds_offset(int row, int g, int s) {
    return (((row >> 5) * 4 + s) * 64 + g * 32 + (row & 31)) * 16;
  }
};
