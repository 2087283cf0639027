// MFMA main loop shared by the projection GEMMs and the LM-head kernel (bf16 models).
//
//   C[M,N] = X[M,K] * W[N,K]^T      X = activations (float16, row-major), W = weights.
//
// Precision.  Weights are bf16 values; activations handed from one operator to the next are kept
// in float16 (11 significant bits) and the products run on the f16 MFMA with float32 accumulation.
// With bf16 (8-bit) activation operands the full-vocabulary logits of a 28-layer decoder drift by
// ~9e-2 from the exact forward; with 11-bit operands they stay near 1e-2.  bf16 weight values
// convert to float16 exactly for 6.1e-5 <= |w| <= 65504 (below that the absolute error is < 6e-8).
//
// Data movement, designed for the verify step's shapes (M = 20..4352 packed rows, weights far
// larger than activations):
//   * Weights are re-packed once (at context creation) into MFMA operand order: for each
//     (32-row tile, 64-wide K tile) a 4 KiB block [s = 0..3][lane = 0..63][8 halves], blocks of one
//     row tile consecutive along K.  A wave streams one or two row tiles: every load instruction
//     reads 1 KiB contiguous, every wave reads a purely sequential stream, and the data land in the
//     operand registers with no LDS hop.  Every weight element is read by exactly one wave of a
//     workgroup, three K tiles deep in flight (register ring).
//   * Activations go through LDS (shared by the 4 waves, which sit side by side along N), stored
//     in fragment order so that each fragment read is one conflict-free 1 KiB ds_read_b128 sweep.
//   * The contraction index inside a K tile is permuted (step s of lane group g multiplies
//     k = 32g + 8s + j) identically for both operands, which is what makes both of the above
//     layouts contiguous.
//   * SWAP = true issues mfma(W, X): the accumulator holds C^T tiles (rows = weight rows, lane =
//     activation row), which makes per-row reductions over N lane-private.
#pragma once
#include "common.h"

typedef _Float16 f16;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;                    // K tile (elements)
constexpr int kWBlock = 32 * kBK;          // elements of one packed (row tile, K tile) block

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ f16x8 as_f16x8(u32x4 v) { return __builtin_bit_cast(f16x8, v); }

// Accumulator element i of lane `lane` in a 32x32 MFMA tile: row, col inside the tile.
__device__ __forceinline__ int acc_row(int lane, int i) { return 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); }
__device__ __forceinline__ int acc_col(int lane) { return lane & 31; }

// Offset (elements) of weight element (n, k) in the packed layout of a matrix with nk K tiles.
__host__ __device__ __forceinline__ size_t packed_w_index(int n, int k, int nk) {
  int nt = n >> 5, nl = n & 31, kt = k >> 6, kk = k & 63;
  int g = kk >> 5, s = (kk & 31) >> 3, j = kk & 7;
  return ((size_t)nt * nk + kt) * kWBlock + (size_t)s * 512 + (g * 32 + nl) * 8 + j;
}

template <int MT, int NT, bool SWAP>
struct MfmaGemm {
  static constexpr int BM = 32 * MT;
  static constexpr int LDS_STAGE_BYTES = MT * 4 * 1024;        // MT row tiles x 4 K-steps x 1 KiB
  static constexpr int LDS_BYTES = 3 * LDS_STAGE_BYTES;        // three stages: see body()

  // Chunk assignment of thread t for the activation tile: chunk q = i*256 + t is the q%8-th 16-byte
  // piece of row q/8, i.e. (g, s) = (q%8 / 4, q%4): eight consecutive lanes read one full 128-byte line
  // of a row.  In LDS the 16-byte slot of (row, g, s) inside its 1 KiB fragment is XOR-swizzled with
  // s + 4g, so that those eight lanes hit eight different bank groups (measured: the unswizzled layout
  // spent 576 LDS conflict cycles per K tile); the fragment reader applies the same permutation and
  // still sweeps its fragment as 64 distinct slots.
  __device__ static __forceinline__ void chunk_of(int i, int& row, int& g, int& s) {
    int q = i * 256 + threadIdx.x;
    row = q >> 3;
    g = (q >> 2) & 1;
    s = q & 3;
  }
  __device__ static __forceinline__ int chunk_lds_offset(int row, int g, int s) {
    return (((row >> 5) * 4 + s) * 64 + ((g * 32 + (row & 31)) ^ (s + 4 * g))) * 16;
  }
  // byte offset of lane `lane`'s slot in fragment (mi, s)
  __device__ static __forceinline__ int frag_lds_offset(int mi, int s, int lane) {
    return ((mi * 4 + s) * 64 + (lane ^ (s + 4 * (lane >> 5)))) * 16;
  }

  struct Operands {
    const f16* x_rows[MT];   // this thread's activation chunks at k = 0 (row and (g, s) offset applied)
    int x_lds[MT];           // byte offset of each chunk inside an LDS stage
    const f16* w_tiles[NT];  // packed weight stream of each row tile at K tile 0, lane offset applied
  };

  template <int STAGE>
  __device__ static __forceinline__ void load_w(u32x4 (&wreg)[3][NT][4], const Operands& op, int kt) {
#pragma unroll
    for (int ni = 0; ni < NT; ++ni)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        wreg[STAGE][ni][s] = *(const u32x4*)(op.w_tiles[ni] + (size_t)kt * kWBlock + s * 512);
      }
  }

  template <int STAGE>
  __device__ static __forceinline__ void load_x(u32x4 (&xreg)[3][MT], const Operands& op, int kt) {
#pragma unroll
    for (int i = 0; i < MT; ++i) xreg[STAGE][i] = *(const u32x4*)(op.x_rows[i] + (size_t)kt * kBK);
  }

  // One K tile.  STAGE = (kt - kt0) % 3 names the ring slots: weights of tile j live in wreg[j % 3], activation
  // chunks of tile j in xreg[j % 3] until they are written to LDS stage j % 3.  Both streams are requested two
  // iterations before they are needed.
  //
  // Issue order.  The MFMA pipe runs asynchronously, so the memory instructions of the iteration are
  // dealt out between the MFMA groups instead of being issued in one burst at the top (14 global loads
  // alone occupy the address path for ~220 cycles during which a one-wave-per-SIMD kernel would leave
  // the matrix unit idle).  Slot j = (K-step s, row tile mi) carries: the LDS read of the fragment
  // needed one K-step later, a share of {LDS store of the next tile's activations, global loads of the
  // activations three tiles ahead, global loads of the weights two tiles ahead}, then the NT MFMAs of
  // (s, mi).  Every load and store is UNCONDITIONAL (tile indices are clamped to the last tile): a
  // prefetch issued under a condition makes the compiler's wait-count tracking assume it may be the
  // newest outstanding load, and the resulting vmcnt(0) waits serialise the ring.
  //
  // The barrier.  The next tile's activations are stored to LDS in the first slots; the workgroup barrier
  // sits between K-steps 2 and 3, and the slots of K-step 3 already read the NEXT tile's step-0 fragments
  // into the free half of xf.  An iteration therefore starts with its first operands in registers: with
  // the barrier at the end of the iteration all four waves hit LDS at once right after it and the matrix
  // unit idled for ~300 cycles per tile until the first fragments arrived.  A wave can now run up to one
  // barrier ahead of the slowest one (storing tile kt+2 while that one still reads tile kt), hence three
  // LDS stages.
  template <int STAGE>
  __device__ static __forceinline__ void body(f32x16 (&acc)[MT][NT], u32x4 (&wreg)[3][NT][4], u32x4 (&xreg)[3][MT],
                                              u32x4 (&xf)[2][MT], const Operands& op, int kt, int kt1, char* lds) {
    const int lane = threadIdx.x & 63;
    constexpr int SLOTS = 4 * MT, EXTRA = 2 * MT + 4 * NT;
    const char* stage = lds + STAGE * LDS_STAGE_BYTES;
    char* nstage = lds + ((STAGE + 1) % 3) * LDS_STAGE_BYTES;
    const int kx = min(kt + 3, kt1 - 1), kw = min(kt + 2, kt1 - 1);
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) {
      const int s = j / MT, mi = j % MT;
      if (j == 3 * MT) {                      // every LDS store of this iteration was issued in an earlier slot
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
      if (s < 3) xf[(s + 1) & 1][mi] = *(const u32x4*)(stage + frag_lds_offset(mi, s + 1, lane));
      else       xf[0][mi] = *(const u32x4*)(nstage + frag_lds_offset(mi, 0, lane));
#pragma unroll
      for (int e = j * EXTRA / SLOTS; e < (j + 1) * EXTRA / SLOTS; ++e) {
        if (e < MT) {
          *(u32x4*)(nstage + op.x_lds[e]) = xreg[(STAGE + 1) % 3][e];
        } else if (e < 2 * MT) {
          xreg[STAGE][e - MT] = *(const u32x4*)(op.x_rows[e - MT] + (size_t)kx * kBK);
        } else {
          const int ni = (e - 2 * MT) / 4, ws = (e - 2 * MT) % 4;
          wreg[(STAGE + 2) % 3][ni][ws] = *(const u32x4*)(op.w_tiles[ni] + (size_t)kw * kWBlock + ws * 512);
        }
      }
      const f16x8 x = as_f16x8(xf[s & 1][mi]);
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) {
        const f16x8 wf = as_f16x8(wreg[STAGE][ni][s]);
        if (SWAP) acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf, x, acc[mi][ni], 0, 0, 0);
        else      acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x, wf, acc[mi][ni], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // Accumulates K tiles [kt0, kt1) into acc.  All 256 threads of the workgroup must call it.  On return the
  // waves are NOT synchronised and LDS may still be read by a slower wave: a caller that reuses LDS puts a
  // barrier first.
  __device__ static __forceinline__ void run(f32x16 (&acc)[MT][NT], const Operands& op, int kt0, int kt1, char* lds) {
    if (kt0 >= kt1) return;
    const int lane = threadIdx.x & 63;
    u32x4 xreg[3][MT];
    u32x4 wreg[3][NT][4];
    u32x4 xf[2][MT];
    load_x<0>(xreg, op, kt0);
    load_w<0>(wreg, op, kt0);
    load_x<1>(xreg, op, min(kt0 + 1, kt1 - 1));
    load_w<1>(wreg, op, min(kt0 + 1, kt1 - 1));
    load_x<2>(xreg, op, min(kt0 + 2, kt1 - 1));
#pragma unroll
    for (int i = 0; i < MT; ++i) *(u32x4*)(lds + op.x_lds[i]) = xreg[0][i];
    __syncthreads();
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) xf[0][mi] = *(const u32x4*)(lds + frag_lds_offset(mi, 0, lane));
    // whole rounds of three tiles without side exits (keeps the register ring free of copies at the
    // back edge), then the one or two remaining tiles
    int kt = kt0;
    for (; kt + 3 <= kt1; kt += 3) {
      body<0>(acc, wreg, xreg, xf, op, kt, kt1, lds);
      body<1>(acc, wreg, xreg, xf, op, kt + 1, kt1, lds);
      body<2>(acc, wreg, xreg, xf, op, kt + 2, kt1, lds);
    }
    if (kt < kt1) {
      body<0>(acc, wreg, xreg, xf, op, kt, kt1, lds);
      if (kt + 1 < kt1) body<1>(acc, wreg, xreg, xf, op, kt + 1, kt1, lds);
    }
  }
};

// ---------------------------------------------------------------------------------------------------------
// Eight-wave variant: a 512-thread workgroup computes a 192-row x 8-weight-row-tile block, its waves arranged
// 2 (rows) x 4 (weight tiles), each holding 96 rows x 2 row tiles (6 accumulator tiles = 96 registers), so two
// waves share every SIMD.  A single wave per SIMD cannot hide the issue cost of its own LDS and global
// instructions behind its MFMAs (measured: a software-pipelined 1 KiB LDS read costs ~17 MFMA cycles, and the
// four-wave loop above runs at ~53 cycles per MFMA against 32 for MFMAs alone); with a second wave on the SIMD the
// matrix unit takes that wave's MFMAs meanwhile.  Measured on the SwiGLU GEMM at M = 576: 59 % instead of 56 % of
// the wave time with the matrix unit busy, 1-3 % less time per launch (no LDS bank conflicts, LDS 35 % busy).  Two
// waves per SIMD leave 256 registers each, too few for a private weight stream as deep as above, so BOTH operands
// go through LDS here: per K tile the workgroup stages 24 KiB of activations and 32 KiB of weights once, and no
// byte is fetched twice by a CU.  The packed weight blocks are already in fragment order: their LDS image is a
// straight copy.
//
// Pipeline per K tile kt (two LDS stages, two register sets): slots 0..6 store the seven 16-byte chunks of tile
// kt + 1 (loaded two iterations ago) to the other stage and immediately reload the same registers with tile
// kt + 3; every slot reads the fragments of the next K-step; the barrier sits before the slots of K-step 3, which
// already read step 0 of tile kt + 1.  Two stages are enough: all reads of a stage are issued (and waited for)
// before the barrier of its own iteration, and it is overwritten only after that barrier.
struct MfmaGemm8 {
  static constexpr int BM = 192, MTW = 3, NTW = 2, THREADS = 512;
  static constexpr int X_STAGE = 6 * 4 * 1024, W_STAGE = 8 * 4096, STAGE_BYTES = X_STAGE + W_STAGE;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;

  struct Operands {
    const char* x_base;      // activation matrix (float16 rows of K elements)
    const char* w_base;      // packed weight matrix
    uint32_t x_off[3];       // byte offset of this thread's activation chunks at k = 0
    int x_lds[3];            // byte offset of each activation chunk inside a stage
    uint32_t w_off[4];       // byte offset of this thread's weight chunks at K tile 0
  };
  // activation chunk i of thread t: q = i*512 + t -> row q/8, (g, s) = (q%8 / 4, q%4)
  __device__ static __forceinline__ void chunk_of(int i, int& row, int& g, int& s) {
    int q = i * 512 + threadIdx.x;
    row = q >> 3;
    g = (q >> 2) & 1;
    s = q & 3;
  }
  __device__ static __forceinline__ int chunk_lds_offset(int row, int g, int s) {
    return (((row >> 5) * 4 + s) * 64 + ((g * 32 + (row & 31)) ^ (s + 4 * g))) * 16;
  }
  __device__ static __forceinline__ int xfrag_offset(int mi_wg, int s, int lane) {
    return ((mi_wg * 4 + s) * 64 + (lane ^ (s + 4 * (lane >> 5)))) * 16;
  }
  // weight chunk i of thread t: LDS tile i*2 + t/256 (= wave column i, row tile t/256 of that wave), 16-byte piece
  // t%256 of its 4 KiB block; the same position inside the stage's weight area
  __device__ static __forceinline__ int w_lds_offset(int i) { return X_STAGE + (i * 2 + (threadIdx.x >> 8)) * 4096 + (threadIdx.x & 255) * 16; }
  __device__ static __forceinline__ int wfrag_offset(int wn, int ni, int s, int lane) {
    return X_STAGE + (wn * 2 + ni) * 4096 + s * 1024 + lane * 16;
  }

  __device__ static __forceinline__ void load_set(u32x4 (&ring)[7], const Operands& op, int kt) {
#pragma unroll
    for (int i = 0; i < 3; ++i) ring[i] = *(const u32x4*)(op.x_base + op.x_off[i] + (size_t)kt * (kBK * 2));
#pragma unroll
    for (int i = 0; i < 4; ++i) ring[3 + i] = *(const u32x4*)(op.w_base + op.w_off[i] + (size_t)kt * (kWBlock * 2));
  }
  __device__ static __forceinline__ void store_chunk(char* stage, const Operands& op, int e, const u32x4& v) {
    if (e < 3) *(u32x4*)(stage + op.x_lds[e]) = v;
    else       *(u32x4*)(stage + w_lds_offset(e - 3)) = v;
  }

  template <int STAGE>
  __device__ static __forceinline__ void body(f32x16 (&acc)[MTW][NTW], u32x4 (&ring)[2][7], u32x4 (&xf)[2][MTW],
                                              u32x4 (&wf)[2][NTW], const Operands& op, int kt, int kt1, char* lds) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const char* stage = lds + STAGE * STAGE_BYTES;
    char* nstage = lds + (1 - STAGE) * STAGE_BYTES;
    const int kl = min(kt + 3, kt1 - 1);
#pragma unroll
    for (int j = 0; j < 12; ++j) {
      const int s = j / 3, mi = j % 3;
      if (j == 9) {
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
      }
      const char* src = (s < 3) ? stage : nstage;
      const int sn = (s + 1) & 3;
      xf[(s + 1) & 1][mi] = *(const u32x4*)(src + xfrag_offset(wm * 3 + mi, sn, lane));
      if (mi < NTW) wf[(s + 1) & 1][mi] = *(const u32x4*)(src + wfrag_offset(wn, mi, sn, lane));
      if (j < 7) {
        store_chunk(nstage, op, j, ring[1 - STAGE][j]);
        if (j < 3) ring[1 - STAGE][j] = *(const u32x4*)(op.x_base + op.x_off[j] + (size_t)kl * (kBK * 2));
        else       ring[1 - STAGE][j] = *(const u32x4*)(op.w_base + op.w_off[j - 3] + (size_t)kl * (kWBlock * 2));
      }
      const f16x8 x = as_f16x8(xf[s & 1][mi]);
#pragma unroll
      for (int ni = 0; ni < NTW; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(wf[s & 1][ni]), x, acc[mi][ni], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // Accumulates K tiles [kt0, kt1) into acc (accumulator tiles hold C^T: rows = weight rows, lane = activation
  // row).  All 512 threads must call it.  On return the waves are not synchronised and LDS may still be read.
  __device__ static __forceinline__ void run(f32x16 (&acc)[MTW][NTW], const Operands& op, int kt0, int kt1, char* lds) {
    if (kt0 >= kt1) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    u32x4 ring[2][7], xf[2][MTW], wf[2][NTW];
    load_set(ring[0], op, kt0);
    load_set(ring[1], op, min(kt0 + 1, kt1 - 1));
#pragma unroll
    for (int e = 0; e < 7; ++e) store_chunk(lds, op, e, ring[0][e]);
    load_set(ring[0], op, min(kt0 + 2, kt1 - 1));
    __syncthreads();
#pragma unroll
    for (int mi = 0; mi < MTW; ++mi) xf[0][mi] = *(const u32x4*)(lds + xfrag_offset(wm * 3 + mi, 0, lane));
#pragma unroll
    for (int ni = 0; ni < NTW; ++ni) wf[0][ni] = *(const u32x4*)(lds + wfrag_offset(wn, ni, 0, lane));
    int kt = kt0;
    for (; kt + 2 <= kt1; kt += 2) {
      body<0>(acc, ring, xf, wf, op, kt, kt1, lds);
      body<1>(acc, ring, xf, wf, op, kt + 1, kt1, lds);
    }
    if (kt < kt1) body<0>(acc, ring, xf, wf, op, kt, kt1, lds);
  }
};
