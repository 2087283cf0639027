// Projection GEMMs of the verify pass (Sec. 3.3 "token-wise" linear layers):
//   QKV (float32 out), O (+residual), gate/up (+SwiGLU), down (+residual).
// bf16 models run on the f16 MFMA main loop of gemm_mfma.h over packed weights; float32 models (the
// tiny parity configuration, launch-latency bound) run on a plain LDS-tiled FMA kernel.
#include "gemm_mfma.h"
#include "gemm_ring2.h"

__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }
// same function with the hardware reciprocal (1 ulp): used in the MFMA epilogue, where a full-precision
// division per output element costs more than the matrix products of a small tile
__device__ __forceinline__ float silu_fast(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// ------------------------------------------------------------------ plain FMA kernel (float32 models)
// 64x64 output tile, K step 16, 256 threads, 4x4 outputs per thread.  For EPI_SWIGLU the tile
// holds gate and up columns of the same 64 output features.
template <typename T, int EPI>
__global__ void __launch_bounds__(256) gemm_simple_kernel(const int32_t* __restrict__ n_rows_dev, int M_max, int N, int K,
                                                          const T* __restrict__ A, const int32_t* __restrict__ a_rows,
                                                          const T* __restrict__ W, void* __restrict__ out) {
  const int M = n_rows_dev ? min(*n_rows_dev, M_max) : M_max;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  if (m0 >= M) return;
  constexpr int NB = (EPI == EPI_SWIGLU) ? 2 : 1;
  __shared__ float sA[16][64 + 1];
  __shared__ float sW[NB][16][64 + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[NB][4][4] = {};
  const int lr = threadIdx.x / 4, lk = (threadIdx.x % 4) * 4;     // loader: row 0..63, k 0,4,8,12
  int arow = min(m0 + lr, M - 1);
  if (a_rows) arow = a_rows[arow];
  const T* ap = A + (size_t)arow * K + lk;
  const int wrow = min(n0 + lr, N - 1);
  const T* wp0 = W + (size_t)wrow * K + lk;
  const T* wp1 = W + (size_t)(wrow + N) * K + lk;                 // up rows (SwiGLU only)
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      sA[lk + j][lr] = to_f32<T>(ap[k0 + j]);
      sW[0][lk + j][lr] = to_f32<T>(wp0[k0 + j]);
      if (NB == 2) sW[NB - 1][lk + j][lr] = to_f32<T>(wp1[k0 + j]);
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], w[NB][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int j = 0; j < 4; ++j) w[nb][j] = sW[nb][kk][tx * 4 + j];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[nb][i][j] = fmaf(a[i], w[nb][j], acc[nb][i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      size_t o = (size_t)m * N + n;
      if (EPI == EPI_STORE) ((T*)out)[o] = from_f32<T>(acc[0][i][j]);
      else if (EPI == EPI_RESID_ADD) ((float*)out)[o] += acc[0][i][j];
      else if (EPI == EPI_SWIGLU) ((T*)out)[o] = from_f32<T>(silu_f(acc[0][i][j]) * acc[NB - 1][i][j]);
      else ((float*)out)[o] = acc[0][i][j];
    }
  }
}

// ------------------------------------------------------------------ weight packing (once per context)
// bf16 row-major [N, K] -> float16 MFMA operand order (see gemm_mfma.h); rows beyond N are zero.
__global__ void __launch_bounds__(256) pack_weight_kernel(const bf16* __restrict__ w, int N, int K, f16* __restrict__ packed,
                                                          size_t n_chunks, int32_t* __restrict__ status) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;     // one 16-byte chunk of the packed array
  if (c >= n_chunks) return;
  const int nk = K / kBK;
  const int lane = c & 63, s = (c >> 6) & 3;
  const size_t blk = c >> 8;
  const int kt = blk % nk, nt = blk / nk;
  const int n = nt * 32 + (lane & 31), k = kt * kBK + (lane >> 5) * 32 + s * 8;
  f16x8 v;
  if (n < N) {
    const bf16x8 src = *(const bf16x8*)(w + (size_t)n * K + k);
    const f16x4 lo = to_f16x4_guarded((float)src[0], (float)src[1], (float)src[2], (float)src[3], status);
    const f16x4 hi = to_f16x4_guarded((float)src[4], (float)src[5], (float)src[6], (float)src[7], status);
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[j] = lo[j]; v[4 + j] = hi[j]; }
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (f16)0.f;
  }
  *(f16x8*)(packed + c * 8) = v;
}

size_t packed_weight_elems(int N, int K) { return (size_t)((N + 31) / 32) * (K / kBK) * kWBlock; }

void launch_pack_weight(const void* w_bf16, int N, int K, void* packed_f16, int32_t* status, hipStream_t st) {
  const size_t n_chunks = packed_weight_elems(N, K) / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((n_chunks + 255) / 256)), dim3(256), 0, st, (const bf16*)w_bf16,
                     N, K, (f16*)packed_f16, n_chunks, status);
}

// ------------------------------------------------------------------ MFMA kernel (bf16 models)
constexpr int kOneRound = 512;    // workgroups that are certainly resident at once (256 CUs, up to two per CU)
// Workgroup tile: BM = 32*MT rows x 4 waves x NT weight row tiles.  For SwiGLU NT == 2 and the two row
// tiles of a wave are the gate rows and the matching up rows of the same 32 output features, so both
// land in the same lane.  Grid: one dimension.  Workgroup ids are dealt round-robin to the 8 XCDs,
// each with its own L2, so the id is decoded XCD-first: the (K split, N block, M block) space, M block
// fastest, is cut into 8 contiguous ranges, one per XCD.  The M blocks that share a weight tile then run back
// to back on one XCD and hit its L2, and an XCD touches one or two K ranges of the activation matrix only
// (measured before this mapping: the down projection fetched 122 MB per launch for 38 MB of operands, every L2
// pulling the whole matrix).
// The float32 epilogues (QKV projection, residual projections) write one partial [M_max, N] slab per K split,
// out[split][m][n]; the consumer (rotary kernel, RMSNorm kernel) sums the slabs.  Float atomics into the
// residual were measured at ~25 us per launch and are not used.
template <int MT, int NT, int EPI>
__global__ void __launch_bounds__(256, (MT <= 3 ? 2 : 1)) gemm_mfma_kernel(const int32_t* __restrict__ n_rows_dev, int M_max, int N, int K,
                                                        const f16* __restrict__ A, const int32_t* __restrict__ a_rows,
                                                        const f16* __restrict__ Wp, void* __restrict__ out,
                                                        int m_blocks, int n_blocks, int n_split, int defer_rows,
                                                        int32_t* __restrict__ status, int adaptive_cap) {
  // accumulators hold C^T tiles (SWAP): a lane owns one activation row and, per group of four
  // registers, four consecutive output columns, so the epilogue stores 8 or 16 bytes per lane
  using G = MfmaGemm<MT, NT, true>;
  extern __shared__ __align__(16) char lds[];
  // The row count lives in device memory.  A launch that fits the chip in one round does not wait for it before
  // its first loads (defer_rows): it reads and multiplies all M_max rows - those at or beyond the count are stale
  // rows of the same buffer, each affecting only its own output row - and applies the count to the stores.  A
  // many-round launch reads it first and skips the row blocks beyond it.
  int M = (!defer_rows && n_rows_dev) ? min(*n_rows_dev, M_max) : M_max;
  if (adaptive_cap > 0) {
    // The launch is sized for the row limit; the row blocks that are live and the number of K splits follow from
    // the step's row count (SlabRule: the consumer of the slabs evaluates the same rule)
    m_blocks = (M + G::BM - 1) / G::BM;
    n_split = gemm_adaptive_split(m_blocks * n_blocks, K / kBK, adaptive_cap);
  }
  // XCD-first decoding: the (split, N block, M block) space, M block fastest, is cut into 8 contiguous ranges,
  // one per XCD (workgroup ids are dealt round-robin to the XCDs)
  const int tiles = m_blocks * n_blocks, total = tiles * n_split;
  const int per_xcd = (total + 7) / 8;
  const int flat = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if ((int)(blockIdx.x / 8) >= per_xcd || flat >= total) return;
  const int split = flat / tiles, id = flat % tiles;
  const int mb = id % m_blocks, nb = id / m_blocks;
  const int m0 = mb * G::BM;
  if (m0 >= M) return;
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  static_assert(!GLU || NT == 2, "SwiGLU pairs one gate tile with one up tile per wave");
  constexpr int NOUT_W = GLU ? 32 : NT * 32;            // output columns per wave
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n_wave0 = (nb * 4 + wave) * NOUT_W;
  const int nk = K / kBK;
  const int n_tiles = (N + 31) / 32;                    // row tiles of the packed matrix (per half for SwiGLU)

  typename G::Operands op;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int row, g, s;
    G::chunk_of(i, row, g, s);
    int r = min(m0 + row, M - 1);
    if (a_rows) r = a_rows[r];
    op.x_rows[i] = A + (size_t)r * K + g * 32 + s * 8;
    op.x_lds[i] = G::chunk_lds_offset(row, g, s);
  }
#pragma unroll
  for (int ni = 0; ni < NT; ++ni) {
    int nt;
    if (GLU) nt = min(n_wave0 / 32, n_tiles - 1) + (ni ? n_tiles : 0);
    else     nt = min(n_wave0 / 32 + ni, n_tiles - 1);
    op.w_tiles[ni] = Wp + (size_t)nt * nk * kWBlock + lane * 8;
  }
  f32x16 acc[MT][NT];
#pragma unroll
  for (int mi = 0; mi < MT; ++mi)
#pragma unroll
    for (int ni = 0; ni < NT; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
  const int kt0 = (int)((long)nk * split / n_split), kt1 = (int)((long)nk * (split + 1) / n_split);
  G::run(acc, op, kt0, kt1, lds);
  if (defer_rows && n_rows_dev) M = min(*n_rows_dev, M_max);

  const int ln = lane & 31, lg = lane >> 5;
#pragma unroll
  for (int mi = 0; mi < MT; ++mi) {
    const int m = m0 + mi * 32 + ln;
    if (m >= M) continue;
    if (GLU) {
      if (n_wave0 >= N) continue;                        // N is a multiple of 32: whole tiles only
      f16* dst = (f16*)out + (size_t)m * N + n_wave0 + 4 * lg;
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        float y[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = silu_fast(acc[mi][0][4 * i4 + j]) * acc[mi][NT - 1][4 * i4 + j];
        *(f16x4*)(dst + 8 * i4) = to_f16x4_guarded(y[0], y[1], y[2], y[3], status);
      }
    } else {
#pragma unroll
      for (int ni = 0; ni < NT; ++ni) {
        const int n0 = n_wave0 + ni * 32;
        if (n0 >= N) continue;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const size_t o = (size_t)m * N + n0 + 8 * i4 + 4 * lg;
          if (EPI == EPI_STORE) {
            *(f16x4*)((f16*)out + o) = to_f16x4_guarded(acc[mi][ni][4 * i4], acc[mi][ni][4 * i4 + 1], acc[mi][ni][4 * i4 + 2],
                                                        acc[mi][ni][4 * i4 + 3], status);
          } else {
            *(f32x4*)((float*)out + (size_t)split * M_max * N + o) =
                f32x4{acc[mi][ni][4 * i4], acc[mi][ni][4 * i4 + 1], acc[mi][ni][4 * i4 + 2], acc[mi][ni][4 * i4 + 3]};
          }
        }
      }
    }
  }
}

template <int MT, int NT, int EPI>
static void launch_mfma(const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const int32_t* a_rows,
                        const void* W, void* out, int n_split, int32_t* status, hipStream_t st) {
  using G = MfmaGemm<MT, NT, true>;
  constexpr int nout = (EPI == EPI_SWIGLU) ? 4 * 32 : 4 * NT * 32;
  int m_blocks = (M_max + G::BM - 1) / G::BM, n_blocks = (N + nout - 1) / nout;
  int total = m_blocks * n_blocks * n_split;
  int grid = 8 * ((total + 7) / 8);
  static bool attr_set = false;              // more than 64 KiB of dynamic LDS needs an opt-in (192-row tiles)
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)gemm_mfma_kernel<MT, NT, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES); attr_set = true; }
  hipLaunchKernelGGL((gemm_mfma_kernel<MT, NT, EPI>), dim3(grid), dim3(256), G::LDS_BYTES, st, n_rows_dev, M_max,
                     N, K, (const f16*)A, a_rows, (const f16*)W, out, m_blocks, n_blocks, n_split, total <= kOneRound ? 1 : 0,
                     status, 0);
}


// Eight-wave kernel (see MfmaGemm8): 192 rows x 128 SwiGLU features (EPI_SWIGLU: gate tile and up tile of the
// same 32 features in one wave) or x 256 output columns (EPI_STORE) per workgroup of 512 threads.
template <int EPI>
__global__ void __launch_bounds__(512) gemm8_kernel(const int32_t* __restrict__ n_rows_dev, int M_max, int N, int K,
                                                    const f16* __restrict__ A, const int32_t* __restrict__ a_rows,
                                                    const f16* __restrict__ Wp, void* __restrict__ out, int m_blocks,
                                                    int n_blocks, int defer_rows, int32_t* __restrict__ status) {
  using G = MfmaGemm8;
  extern __shared__ __align__(16) char lds[];
  int M = (!defer_rows && n_rows_dev) ? min(*n_rows_dev, M_max) : M_max;     // see gemm_mfma_kernel
  const int total = m_blocks * n_blocks, per_xcd = (total + 7) / 8;
  const int id = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if ((int)(blockIdx.x / 8) >= per_xcd || id >= total) return;
  const int mb = id % m_blocks, nb = id / m_blocks;
  const int m0 = mb * G::BM;
  if (m0 >= M) return;
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = wave >> 2, wn = wave & 3;
  const int nk = K / kBK;
  const int n_tiles = (N + 31) / 32;

  G::Operands op;
  op.x_base = (const char*)A;
  op.w_base = (const char*)Wp;
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    int row, g, s;
    G::chunk_of(i, row, g, s);
    int r = min(m0 + row, M - 1);
    if (a_rows) r = a_rows[r];
    op.x_off[i] = (uint32_t)(((size_t)r * K + g * 32 + s * 8) * 2);
    op.x_lds[i] = G::chunk_lds_offset(row, g, s);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ni = threadIdx.x >> 8;
    int nt;
    if (GLU) nt = min(nb * 4 + i, n_tiles - 1) + ni * n_tiles;
    else     nt = min(nb * 8 + i * 2 + ni, n_tiles - 1);
    op.w_off[i] = (uint32_t)(((size_t)nt * nk * kWBlock + (threadIdx.x & 255) * 8) * 2);
  }
  f32x16 acc[3][2];
#pragma unroll
  for (int mi = 0; mi < 3; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
    G::run(acc, op, 0, nk, lds);
  if (defer_rows && n_rows_dev) M = min(*n_rows_dev, M_max);

  const int ln = lane & 31, lg = lane >> 5;
  const int n_wave0 = GLU ? (nb * 4 + wn) * 32 : (nb * 4 + wn) * 64;
#pragma unroll
  for (int mi = 0; mi < 3; ++mi) {
    const int m = m0 + wm * 96 + mi * 32 + ln;
    if (m >= M) continue;
    if (GLU) {
      if (n_wave0 >= N) continue;
      f16* dst = (f16*)out + (size_t)m * N + n_wave0 + 4 * lg;
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        float y[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = silu_fast(acc[mi][0][4 * i4 + j]) * acc[mi][1][4 * i4 + j];
        *(f16x4*)(dst + 8 * i4) = to_f16x4_guarded(y[0], y[1], y[2], y[3], status);
      }
    } else {
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int n0 = n_wave0 + ni * 32;
        if (n0 >= N) continue;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *(f16x4*)((f16*)out + (size_t)m * N + n0 + 8 * i4 + 4 * lg) =
              to_f16x4_guarded(acc[mi][ni][4 * i4], acc[mi][ni][4 * i4 + 1], acc[mi][ni][4 * i4 + 2], acc[mi][ni][4 * i4 + 3], status);
      }
    }
  }
}

// Large-batch kernels (row limit above 640) on the MfmaGemmRing2 loop: 128 rows x 8 weight row tiles per workgroup,
// two workgroups per CU.  The row count is read first (these launches run several rounds of the CUs) and row blocks
// beyond it exit.
//
// SwiGLU: wave w holds the gate tile and the up tile of features 32 w .. 32 w + 31 of the block's 128 features.
__global__ void __launch_bounds__(256, 2) gemm_ring2_swiglu_kernel(const int32_t* __restrict__ n_rows_dev, int M_max, int N, int K,
                                                                  const f16* __restrict__ A, const f16* __restrict__ Wp,
                                                                  f16* __restrict__ out, int m_blocks, int n_blocks,
                                                                  int32_t* __restrict__ status) {
  using G = MfmaGemmRing2;
  extern __shared__ __align__(16) char lds[];
  const int M = min(*n_rows_dev, M_max);
  const int total = m_blocks * n_blocks, per_xcd = (total + 7) / 8;
  const int id = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;      // XCD-first decoding, M block fastest
  if ((int)(blockIdx.x / 8) >= per_xcd || id >= total) return;
  const int mb = id % m_blocks, nb = id / m_blocks;
  const int m0 = mb * G::BM;
  if (m0 >= M) return;
  // the wave index is made scalar so that the weight stream's base address stays on the scalar unit
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int nk = K / kBK;
  const int n_tiles = (N + 31) / 32;                    // row tiles of each half of the packed gate/up matrix
  const int n_wave0 = (nb * 4 + wave) * 32;
  const int gate_tile = min(n_wave0 / 32, n_tiles - 1);
  const int ln = lane & 31, lg = lane >> 5;
  // the last row block of a step with at most 64 live rows computes two row tiles instead of four
  auto tile = [&](auto mt_tag) {
    constexpr int MT = decltype(mt_tag)::value;
    using GT = MfmaGemmRing2T<MT>;
    typename GT::Operands op;
    GT::make_operands(op, A, K, m0, M, Wp, nk, gate_tile, gate_tile + n_tiles);
    f32x16 acc[MT][2];
#pragma unroll
    for (int mi = 0; mi < MT; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
    GT::run(acc, op, 0, nk, lds);
    if (n_wave0 >= N) return;                           // N is a multiple of 32: whole tiles only
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
      const int m = m0 + mi * 32 + ln;
      if (m >= M) continue;
      f16* dst = out + (size_t)m * N + n_wave0 + 4 * lg;
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        float y[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = silu_fast(acc[mi][0][4 * i4 + j]) * acc[mi][1][4 * i4 + j];
        *(f16x4*)(dst + 8 * i4) = to_f16x4_guarded(y[0], y[1], y[2], y[3], status);
      }
    }
  };
  if (M - m0 <= 64) tile(std::integral_constant<int, 2>{});
  else tile(std::integral_constant<int, 4>{});
}

// Residual projections above 640 rows, 256 output columns per workgroup, float32 K-split slabs.  The row tile (96
// rows on the MfmaGemm<3, 2> loop or 128 rows on the MfmaGemmRing2 loop), the live row blocks and the number of K
// splits all follow from the step's row count (SlabRule: the consumer of the slabs evaluates the same rule): which
// tile fills the 512 resident workgroup slots better depends on the row count, which only the device knows
// (measured, down projection: 7B shape at 1185 rows, 96-row tiles 2 x 182 workgroups 194 us, 128-row tiles 3 x 140
// workgroups 172 us; 1.5B shape at 3952 rows, 96-row tiles 2 x 252 workgroups 108 us, 128-row tiles 2 x 186 120 us).
__global__ void __launch_bounds__(256, 2) gemm_resid_kernel(const int32_t* __restrict__ n_rows_dev, int M_max, int N, int K,
                                                           const f16* __restrict__ A, const f16* __restrict__ Wp,
                                                           float* __restrict__ out, SlabRule rule) {
  extern __shared__ __align__(16) char lds[];
  const int M = min(*n_rows_dev, M_max);
  const int bm = rule.tile_rows(M);
  const int m_blocks = (M + bm - 1) / bm, tiles = m_blocks * rule.n_blocks;
  const int nk = rule.nk;
  const int n_split = gemm_adaptive_split(tiles, nk, rule.cap);
  // XCD-first decoding: the (split, N block, M block) space, M block fastest, is cut into 8 contiguous ranges
  const int total = tiles * n_split, per_xcd = (total + 7) / 8;
  const int flat = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if ((int)(blockIdx.x / 8) >= per_xcd || flat >= total) return;
  const int split = flat / tiles, id = flat % tiles;
  const int mb = id % m_blocks, nb = id / m_blocks;
  const int m0 = mb * bm;
  // the wave index is made scalar so that the weight stream's base address stays on the scalar unit
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int ln = lane & 31, lg = lane >> 5;
  const int n_tiles = (N + 31) / 32;
  const int n_wave0 = (nb * 4 + wave) * 64;
  const int tile0 = min(n_wave0 / 32, n_tiles - 1), tile1 = min(n_wave0 / 32 + 1, n_tiles - 1);
  const int kt0 = (int)((long)nk * split / n_split), kt1 = (int)((long)nk * (split + 1) / n_split);
  float* dst = out + (size_t)split * M_max * N;
  auto store = [&](auto& acc, auto mt_tag) {
    constexpr int MT = decltype(mt_tag)::value;
#pragma unroll
    for (int mi = 0; mi < MT; ++mi) {
      const int m = m0 + mi * 32 + ln;
      if (m >= M) continue;
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) {
        const int n0 = n_wave0 + ni * 32;
        if (n0 >= N) continue;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *(f32x4*)(dst + (size_t)m * N + n0 + 8 * i4 + 4 * lg) =
              f32x4{acc[mi][ni][4 * i4], acc[mi][ni][4 * i4 + 1], acc[mi][ni][4 * i4 + 2], acc[mi][ni][4 * i4 + 3]};
      }
    }
  };
  if (bm == MfmaGemmRing2::BM) {
    using G = MfmaGemmRing2;
    G::Operands op;
    G::make_operands(op, A, K, m0, M, Wp, nk, tile0, tile1);
    f32x16 acc[4][2];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
    G::run(acc, op, kt0, kt1, lds);
    store(acc, std::integral_constant<int, 4>{});
  } else {
    using G = MfmaGemm<3, 2, true>;
    typename G::Operands op;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      int row, g, s;
      G::chunk_of(i, row, g, s);
      const int r = min(m0 + row, M - 1);
      op.x_rows[i] = A + (size_t)r * K + g * 32 + s * 8;
      op.x_lds[i] = G::chunk_lds_offset(row, g, s);
    }
    op.w_tiles[0] = Wp + (size_t)tile0 * nk * kWBlock + lane * 8;
    op.w_tiles[1] = Wp + (size_t)tile1 * nk * kWBlock + lane * 8;
    f32x16 acc[3][2];
#pragma unroll
    for (int mi = 0; mi < 3; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
    G::run(acc, op, kt0, kt1, lds);
    store(acc, std::integral_constant<int, 3>{});
  }
}

// The ring2 kernels address the activation matrix with 32-bit byte offsets.
static bool ring2_applies(int M_max, int K) { return (size_t)M_max * K * 2 < ((size_t)1 << 32); }

static void launch_ring2_swiglu(const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const void* W, void* out,
                                int32_t* status, hipStream_t st) {
  using G = MfmaGemmRing2;
  const int m_blocks = (M_max + G::BM - 1) / G::BM, n_blocks = (N + 127) / 128;
  const int grid = 8 * ((m_blocks * n_blocks + 7) / 8);
  hipLaunchKernelGGL(gemm_ring2_swiglu_kernel, dim3(grid), dim3(256), G::LDS_BYTES, st, n_rows_dev, M_max, N, K, (const f16*)A,
                     (const f16*)W, (f16*)out, m_blocks, n_blocks, status);
}

template <int EPI>
static void launch_gemm8(const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const int32_t* a_rows,
                         const void* W, void* out, int32_t* status, hipStream_t st) {
  using G = MfmaGemm8;
  constexpr int nout = (EPI == EPI_SWIGLU) ? 128 : 256;
  const int m_blocks = (M_max + G::BM - 1) / G::BM, n_blocks = (N + nout - 1) / nout;
  const int grid = 8 * ((m_blocks * n_blocks + 7) / 8);
  static bool attr_set = false;
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)gemm8_kernel<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES); attr_set = true; }
  hipLaunchKernelGGL((gemm8_kernel<EPI>), dim3(grid), dim3(512), G::LDS_BYTES, st, n_rows_dev, M_max, N, K,
                     (const f16*)A, a_rows, (const f16*)W, out, m_blocks, n_blocks, m_blocks * n_blocks <= kOneRound ? 1 : 0, status);
}

// The eight-wave kernel addresses both matrices with 32-bit byte offsets and pays off when 192-row blocks fit
// the row count without much padding.
static bool gemm8_applies(int M_max, int N, int K, int w_rows) {
  if ((size_t)M_max * K * 2 >= ((size_t)1 << 32) || packed_weight_elems(w_rows, K) * 2 >= ((size_t)1 << 32)) return false;
  const int pad6 = (M_max + 191) / 192 * 192, pad4 = (M_max + 127) / 128 * 128;
  return M_max > 128 && pad6 <= pad4;
}

template <typename T, int EPI>
static void launch_simple(const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const int32_t* a_rows,
                          const void* W, void* out, hipStream_t st) {
  dim3 grid((N + 63) / 64, (M_max + 63) / 64);
  hipLaunchKernelGGL((gemm_simple_kernel<T, EPI>), grid, dim3(256), 0, st, n_rows_dev, M_max, N, K, (const T*)A, a_rows,
                     (const T*)W, out);
}

// Tile choice.  MT: smallest row tiling that covers M_max with the least padding (576 rows -> 3 x 192).
// NT: two row tiles per wave (256 columns per workgroup) when that still yields enough workgroups for
// 256 CUs, else one.  K split (residual epilogue only) when even that leaves most CUs idle.
static int pick_mt(int M_max) {
  if (M_max <= 32) return 1;
  if (M_max <= 64) return 2;
  if (M_max <= 128) return 4;
  const int pad6 = (M_max + 191) / 192 * 192, pad4 = (M_max + 127) / 128 * 128;
  return pad6 <= pad4 ? 6 : 4;
}

template <int EPI>
static int dispatch(int dtype, const int32_t* n_rows_dev, int M_max, int N, int K, const void* A,
                    const int32_t* a_rows, const void* W, void* out, int32_t* status, hipStream_t st) {
  if (dtype == BS_F32) { launch_simple<float, EPI>(n_rows_dev, M_max, N, K, A, a_rows, W, out, st); return 0; }
  bool small_tiles = false;
  if constexpr (EPI == EPI_SWIGLU) {
    // large batches: 128-row tiles on the in-place two-tile ring (see gemm_ring2.h), two workgroups per CU
    // (measured against the 96-row tiles below: 7B shape at 1185 rows 316 -> 302 us, 1.5B shape at 3952 rows 220 -> 216)
    if (M_max > 640 && n_rows_dev && !a_rows && ring2_applies(M_max, K)) {
      launch_ring2_swiglu(n_rows_dev, M_max, N, K, A, W, out, status, st);
      return 1;
    }
    bool want = true;
    if (M_max > 128) {
      // 192-row tiles, one workgroup per CU, against 96-row tiles, two per CU: whichever needs less time by rounds of
      // the 256 CUs.  In a single round the small tiles are about 10 % slower per unit of work; over several rounds
      // they are faster, because one workgroup's pipeline fill and epilogue overlap the other's main loop.
      // Measured, 7B shape (18944 features): 288 rows, 2 x 148 workgroups = two rounds against 3 x 148 small ones at
      // once: 133 -> 96 us; 1152 rows, 3.5 rounds either way: 308 -> 290 us.
      const int nb = (N + 127) / 128;
      const long r6 = ((M_max + 191) / 192 * nb + 255) / 256, r3 = ((M_max + 95) / 96 * nb + 511) / 512;
      const long cost6 = r6 * 60, cost3 = r3 * (r3 > 1 ? 57 : 66);
      if (cost3 < cost6) { want = false; small_tiles = true; }
    }
    if (want && gemm8_applies(M_max, N, K, 2 * N)) {
      launch_gemm8<EPI>(n_rows_dev, M_max, N, K, A, a_rows, W, out, status, st);
      return 1;
    }
  }
  int mt = small_tiles ? 3 : pick_mt(M_max);
  // float32-epilogue GEMMs have narrow outputs (N = d or Nqkv): measured on MI355X at M = 576, smaller row
  // tiles with at most 4 K splits beat 192-row tiles with 7 splits (down projection 50 -> 33 us, O 17 -> 13 us)
  if ((EPI == EPI_RESID_ADD || EPI == EPI_STORE_F32) && M_max > 64) mt = (K / kBK <= 32) ? 2 : 4;
  const int m_blocks = (M_max + mt * 32 - 1) / (mt * 32);
  int nt = 2;
  if (EPI != EPI_SWIGLU) {
    // 256-column tiles (two weight row tiles per wave: half the LDS reads per MFMA) if they can fill the chip, for
    // the float32 epilogues with the help of two K splits (more slabs would cost the consumer more than the tiles
    // gain; 7B shape, 1152 rows, down projection: 126 tiles x 2 splits take 147 us, 252 tiles of 128 columns 172 us)
    int blocks2 = m_blocks * ((N + 255) / 256);
    if (EPI == EPI_RESID_ADD || EPI == EPI_STORE_F32) {
      int s2 = (256 + blocks2 / 2) / blocks2;
      if (s2 > K / kBK / 4) s2 = K / kBK / 4;
      if (s2 > 2) s2 = 2;
      if (s2 > 1) blocks2 *= s2;
    }
    if (blocks2 < 200) nt = 1;
  }
  const int nout = (EPI == EPI_SWIGLU) ? 128 : nt * 128;
  const int blocks = m_blocks * ((N + nout - 1) / nout);
  int n_split = 1;
  if (EPI == EPI_RESID_ADD || EPI == EPI_STORE_F32) {
    const int nk = K / kBK;
    if (blocks < 160) n_split = (256 + blocks / 2) / blocks;
    if (n_split > nk / 4) n_split = nk / 4 > 0 ? nk / 4 : 1;       // at least 4 K tiles per split
    if (n_split < 1) n_split = 1;
    if (n_split > 4) n_split = 4;
    if (n_split > nk) n_split = nk;
  }
#define BS_GEMM(MT_, NT_) launch_mfma<MT_, NT_, EPI>(n_rows_dev, M_max, N, K, A, a_rows, W, out, n_split, status, st)
  if constexpr (EPI != EPI_SWIGLU) {
    if (nt == 1) {
      switch (mt) { case 1: BS_GEMM(1, 1); break; case 2: BS_GEMM(2, 1); break; case 3: BS_GEMM(3, 1); break; case 4: BS_GEMM(4, 1); break; default: BS_GEMM(6, 1); }
      return n_split;
    }
  }
  switch (mt) { case 1: BS_GEMM(1, 2); break; case 2: BS_GEMM(2, 2); break; case 3: BS_GEMM(3, 2); break; case 4: BS_GEMM(4, 2); break; default: BS_GEMM(6, 2); }
#undef BS_GEMM
  return n_split;
}

// Residual projections (O, down): float32 K-split slabs, summed into the residual by the next RMSNorm.
// Above 64 rows: 96-row tiles, two workgroups per CU, 256 output columns per workgroup when the row limit gives
// enough of them (else 128), and the number of K splits decided on the device from the step's row count: with the
// split fixed for the row limit B (k_max + 1), a ragged step (1185 of at most 2176 rows, 7B shape) ran the down
// projection as 140 live workgroups of 128 x 256 on 256 CUs, 239 us; one resident round of 2 x 182 takes 189 us.
template <int NT>
static SlabRule launch_resid_adaptive(const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const void* W,
                                      void* out, int32_t* status, hipStream_t st) {
  using G = MfmaGemm<3, NT, true>;
  constexpr int nout = 4 * NT * 32, cap = 512;
  const int m_blocks = (M_max + G::BM - 1) / G::BM, n_blocks = (N + nout - 1) / nout, nk = K / kBK;
  const int tiles_max = m_blocks * n_blocks;
  const int grid = 8 * (((tiles_max > cap ? tiles_max : cap) + 7) / 8);     // tiles(M) * splits(M) never exceeds this
  static bool attr_set = false;
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)gemm_mfma_kernel<3, NT, EPI_RESID_ADD>, hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES); attr_set = true; }
  hipLaunchKernelGGL((gemm_mfma_kernel<3, NT, EPI_RESID_ADD>), dim3(grid), dim3(256), G::LDS_BYTES, st, n_rows_dev, M_max, N, K,
                     (const f16*)A, nullptr, (const f16*)W, out, m_blocks, n_blocks, 1, 0, status, cap);
  return SlabRule{0, G::BM, n_blocks, nk, cap, 0};
}

SlabRule launch_gemm_resid(int dtype, const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const void* W,
                           void* out, int32_t* status, hipStream_t st) {
  // (up to 640 rows the fixed launches below are tuned for one resident round and start their loads before the row
  // count arrives; measured at 576 rows, 1.5B shape, the device-side rule costs the down projection 22 -> 27 us)
  if (dtype == BS_BF16 && M_max > 640 && n_rows_dev) {
    const int tiles2 = (M_max + 95) / 96 * ((N + 255) / 256);
    if (tiles2 >= 128) {
      constexpr int cap = 512;
      const bool dual = ring2_applies(M_max, K);
      const int n_blocks = (N + 255) / 256, nk = K / kBK;
      const int tiles_max = (M_max + 95) / 96 * n_blocks;                      // the smaller tile gives more of them
      const int grid = 8 * (((tiles_max > cap ? tiles_max : cap) + 7) / 8);   // tiles(M) * splits(M) never exceeds this
      const SlabRule rule{0, 96, n_blocks, nk, cap, dual ? MfmaGemmRing2::BM : 0};
      constexpr int lds = MfmaGemm<3, 2, true>::LDS_BYTES > MfmaGemmRing2::LDS_BYTES ? MfmaGemm<3, 2, true>::LDS_BYTES : MfmaGemmRing2::LDS_BYTES;
      hipLaunchKernelGGL(gemm_resid_kernel, dim3(grid), dim3(256), lds, st, n_rows_dev, M_max, N, K, (const f16*)A,
                         (const f16*)W, (float*)out, rule);
      return rule;
    }
    return launch_resid_adaptive<1>(n_rows_dev, M_max, N, K, A, W, out, status, st);
  }
  const int n = launch_gemm(dtype, EPI_RESID_ADD, n_rows_dev, M_max, N, K, A, nullptr, W, out, status, st);
  return SlabRule{n, 0, 0, 0, 0, 0};
}

int launch_gemm(int dtype, GemmEpilogue epi, const int32_t* n_rows_dev, int M_max, int N, int K, const void* A,
                const int32_t* a_rows, const void* W, void* out, int32_t* status, hipStream_t st) {
  switch (epi) {
    case EPI_STORE: return dispatch<EPI_STORE>(dtype, n_rows_dev, M_max, N, K, A, a_rows, W, out, status, st);
    case EPI_RESID_ADD: return dispatch<EPI_RESID_ADD>(dtype, n_rows_dev, M_max, N, K, A, a_rows, W, out, status, st);
    case EPI_SWIGLU: return dispatch<EPI_SWIGLU>(dtype, n_rows_dev, M_max, N, K, A, a_rows, W, out, status, st);
    default: return dispatch<EPI_STORE_F32>(dtype, n_rows_dev, M_max, N, K, A, a_rows, W, out, status, st);
  }
}
