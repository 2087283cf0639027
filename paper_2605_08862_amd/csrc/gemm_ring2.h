// Main loop for the large-batch GEMMs (row limit above 640): a four-wave workgroup computes 128 rows x 8 weight row
// tiles, every wave all 128 rows (four row tiles) x its own two weight row tiles (8 accumulator tiles = 128
// registers), two workgroups per CU.
//
// Why this shape.  The loop of MfmaGemm<3, 2> (96 rows, two workgroups per CU) is limited by the path from L2 into
// the CU: per 64-wide K tile a workgroup pulls 12 KiB of activations and 32 KiB of weights through the texture
// addresser for 3.1 MFLOP, which is 57 bytes per clock per CU at full matrix rate against a nominal 64 (measured
// there: addresser busy 80 % of the time, matrix unit 56 %).  A 128-row tile needs 16 + 32 KiB for 4.2 MFLOP, 47
// bytes per clock.  What kept MfmaGemm from it is registers: 128 accumulator registers, a three-tile weight ring
// (96) and double-buffered fragments (32) do not leave room for two waves per SIMD.  Here
//   * the weight ring holds TWO K tiles and is refilled in place: the fragments of K-step s are requested for tile
//     kt + 2 right after the last MFMA of step s of tile kt has been issued (64 registers, loads still in flight for
//     almost two tiles);
//   * each activation fragment register is refilled from LDS with the same row tile's fragment of the next K-step
//     right after its own MFMAs (16 registers; the three other row tiles' MFMAs cover the LDS latency);
//   * the activation chunks use one register set, stored to LDS one tile after they were requested, and two LDS
//     stages (the barrier sits before K-step 3, when every read of the current stage has been issued and waited for,
//     so the stage of tile kt - 1 is free for tile kt + 1: see MfmaGemm8).
// Measured on MI355X, gate/up projection: 7B shape at 1185 rows 316 -> 302 us, 1.5B shape at 3952 rows 220 -> 216 us.
// Measured and dropped: the same loop with eight waves in one workgroup (128 rows x 16 weight row tiles, activations
// fetched once for all eight: 40 bytes per clock) runs 357 / 225 us: both waves of a SIMD then belong to one
// workgroup and meet the same barrier, so their stalls coincide instead of filling each other's gaps; raising or
// lowering the wave priority around the MFMAs (s_setprio) costs 45 %.
#pragma once
#include "gemm_mfma.h"

// MT_ = 4 is the tile the launchers count with; MT_ = 2 computes only the upper 64 rows of such a tile (the last row
// block of a step when at most 64 of its rows are live).
template <int MT_>
struct MfmaGemmRing2T {
  static constexpr int MT = MT_, NT = 2, BM = 32 * MT, THREADS = 256, NCH = MT;
  static constexpr int STAGE_BYTES = MT * 4 * 1024;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int CHUNK_LDS_STEP = 4096;   // chunk i of a thread lies 32 rows (one row tile) further down

  struct Operands {
    const char* x_base;        // activation matrix (uniform)
    uint32_t x_off[NCH];       // byte offset of this thread's activation chunks at k = 0 (row and (g, s) applied)
    int x_lds;                 // byte offset of chunk 0 inside an LDS stage; chunk i lies i * CHUNK_LDS_STEP further
    const char* w_base[NT];    // packed weight stream of the wave's row tiles at K tile 0 (uniform within the wave)
    uint32_t w_lane;           // byte offset of this lane inside a 1 KiB fragment
  };
  // activation chunk i of thread t: q = i*256 + t -> row q/8 = 32 i + t/8, (g, s) = (q%8 / 4, q%4)
  __device__ static __forceinline__ void chunk_of(int i, int& row, int& g, int& s) {
    const int q = i * THREADS + threadIdx.x;
    row = q >> 3;
    g = (q >> 2) & 1;
    s = q & 3;
  }
  __device__ static __forceinline__ int chunk_lds_offset(int row, int g, int s) {
    return (((row >> 5) * 4 + s) * 64 + ((g * 32 + (row & 31)) ^ (s + 4 * g))) * 16;
  }
  __device__ static __forceinline__ int frag_lds_offset(int mi, int s, int lane) {
    return ((mi * 4 + s) * 64 + (lane ^ (s + 4 * (lane >> 5)))) * 16;
  }

  template <int STAGE>
  __device__ static __forceinline__ void body(f32x16 (&acc)[MT][NT], u32x4 (&wreg)[2][NT][4], u32x4 (&xreg)[NCH],
                                              u32x4 (&xf)[MT], const Operands& op, int kt, int kt1, char* lds) {
    const int lane = threadIdx.x & 63;
    const char* stage = lds + STAGE * STAGE_BYTES;
    char* nstage = lds + (1 - STAGE) * STAGE_BYTES;
    const int kx = min(kt + 2, kt1 - 1), kw = min(kt + 2, kt1 - 1);    // every prefetch unconditional, clamped
#pragma unroll
    for (int j = 0; j < 4 * MT; ++j) {
      const int s = j / MT, mi = j % MT;
      if (j == 3 * MT) {                      // the stores of tile kt + 1 were issued in slots 0 .. 3
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
      if (j < NCH) {
        *(u32x4*)(nstage + op.x_lds + j * CHUNK_LDS_STEP) = xreg[j];
        xreg[j] = *(const u32x4*)(op.x_base + op.x_off[j] + (size_t)kx * (kBK * 2));
      }
      const f16x8 x = as_f16x8(xf[mi]);
#pragma unroll
      for (int ni = 0; ni < NT; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(wreg[STAGE][ni][s]), x, acc[mi][ni], 0, 0, 0);
      // the fragment just used makes room for the same row tile's fragment of the next K-step (after the barrier:
      // step 0 of the next tile)
      xf[mi] = *(const u32x4*)((s < 3 ? stage : nstage) + frag_lds_offset(mi, (s + 1) & 3, lane));
      if (mi == MT - 1) {
#pragma unroll
        for (int ni = 0; ni < NT; ++ni)
          wreg[STAGE][ni][s] = *(const u32x4*)(op.w_base[ni] + (size_t)kw * (kWBlock * 2) + s * 1024 + op.w_lane);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // Accumulates K tiles [kt0, kt1) into acc (C^T tiles: rows = weight rows, lane = activation row).  All 256
  // threads must call it.  On return the waves are not synchronised and LDS may still be read.
  __device__ static __forceinline__ void run(f32x16 (&acc)[MT][NT], const Operands& op, int kt0, int kt1, char* lds) {
    if (kt0 >= kt1) return;
    const int lane = threadIdx.x & 63;
    u32x4 xreg[NCH], wreg[2][NT][4], xf[MT];
    const int k1 = min(kt0 + 1, kt1 - 1);
#pragma unroll
    for (int i = 0; i < NCH; ++i) xreg[i] = *(const u32x4*)(op.x_base + op.x_off[i] + (size_t)kt0 * (kBK * 2));
#pragma unroll
    for (int ni = 0; ni < NT; ++ni)
#pragma unroll
      for (int s = 0; s < 4; ++s) wreg[0][ni][s] = *(const u32x4*)(op.w_base[ni] + (size_t)kt0 * (kWBlock * 2) + s * 1024 + op.w_lane);
#pragma unroll
    for (int ni = 0; ni < NT; ++ni)
#pragma unroll
      for (int s = 0; s < 4; ++s) wreg[1][ni][s] = *(const u32x4*)(op.w_base[ni] + (size_t)k1 * (kWBlock * 2) + s * 1024 + op.w_lane);
#pragma unroll
    for (int i = 0; i < NCH; ++i) *(u32x4*)(lds + op.x_lds + i * CHUNK_LDS_STEP) = xreg[i];
#pragma unroll
    for (int i = 0; i < NCH; ++i) xreg[i] = *(const u32x4*)(op.x_base + op.x_off[i] + (size_t)k1 * (kBK * 2));
    __syncthreads();
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) xf[mi] = *(const u32x4*)(lds + frag_lds_offset(mi, 0, lane));
    int kt = kt0;
    for (; kt + 2 <= kt1; kt += 2) {
      body<0>(acc, wreg, xreg, xf, op, kt, kt1, lds);
      body<1>(acc, wreg, xreg, xf, op, kt + 1, kt1, lds);
    }
    if (kt < kt1) body<0>(acc, wreg, xreg, xf, op, kt, kt1, lds);
  }

  // Operands of a workgroup tile: rows m0 .. m0 + BM - 1 of A (clamped to the last live row M - 1), weight row tiles
  // tile0 and tile1 of the packed matrix for this wave.
  __device__ static __forceinline__ void make_operands(Operands& op, const f16* A, int K, int m0, int M, const f16* Wp,
                                                       int nk, int tile0, int tile1) {
    op.x_base = (const char*)A;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int row, g, s;
      chunk_of(i, row, g, s);
      const int r = min(m0 + row, M - 1);
      op.x_off[i] = (uint32_t)(((size_t)r * K + g * 32 + s * 8) * 2);
      if (i == 0) op.x_lds = chunk_lds_offset(row, g, s);
    }
    op.w_base[0] = (const char*)(Wp + (size_t)tile0 * nk * kWBlock);
    op.w_base[1] = (const char*)(Wp + (size_t)tile1 * nk * kWBlock);
    op.w_lane = (threadIdx.x & 63) * 16;
  }
};
using MfmaGemmRing2 = MfmaGemmRing2T<4>;
