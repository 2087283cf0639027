// Projection GEMMs of the verify pass (Sec. 3.3 "token-wise" linear layers):
//   QKV, O (+residual), gate/up (+SwiGLU), down (+residual), and plain float32 stores.
// bf16 models run on the MFMA main loop of gemm_mfma.h; float32 models (the tiny parity
// configuration, launch-latency bound) run on a plain LDS-tiled FMA kernel.
#include "gemm_mfma.h"
#include <stdlib.h>

// ------------------------------------------------------------------ epilogue helpers
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// ------------------------------------------------------------------ plain FMA kernel (any dtype)
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

// ------------------------------------------------------------------ MFMA kernel (bf16)
// Workgroup tile: BM = 32*MT rows x BNW = 4*NT*32 weight rows (for SwiGLU: half of them are gate
// rows, the other half the matching up rows, interleaved per 32 so that accumulators [..][2j] and
// [..][2j+1] of one lane hold gate and up of the same output feature).
// Block order: ids are dealt round-robin to the 8 XCDs by the hardware; remap so that the M
// blocks that share one weight tile run on the same XCD back to back and hit its L2.
template <int MT, int NT, int EPI>
__global__ void __launch_bounds__(256) gemm_mfma_kernel(const int32_t* __restrict__ n_rows_dev, int M_max, int N, int K,
                                                        const bf16* __restrict__ A, const int32_t* __restrict__ a_rows,
                                                        const bf16* __restrict__ W, void* __restrict__ out,
                                                        int m_blocks, int n_blocks) {
  using G = MfmaGemm<MT, NT, false>;
  extern __shared__ __align__(16) char lds[];
  const int M = n_rows_dev ? min(*n_rows_dev, M_max) : M_max;
  const int total = m_blocks * n_blocks;
  const int per_xcd = (total + 7) / 8;
  const int id = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (id >= total) return;
  const int mb = id % m_blocks, nb = id / m_blocks;
  const int m0 = mb * G::BM;
  if (m0 >= M) return;
  constexpr bool GLU = (EPI == EPI_SWIGLU);
  constexpr int NOUT_W = GLU ? NT * 16 : NT * 32;       // output columns per wave
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n_wave0 = nb * 4 * NOUT_W + wave * NOUT_W;

  const bf16* x_rows[MT];
  int x_lds[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int row, g, s;
    G::chunk_of(i, row, g, s);
    int r = min(m0 + row, M - 1);
    if (a_rows) r = a_rows[r];
    x_rows[i] = A + (size_t)r * K + g * 32 + s * 8;
    x_lds[i] = G::chunk_lds_offset(row, g, s);
  }
  const bf16* w_rows[NT];
#pragma unroll
  for (int ni = 0; ni < NT; ++ni) {
    int n;
    if (GLU) n = min(n_wave0 + (ni >> 1) * 32 + (lane & 31), N - 1) + ((ni & 1) ? N : 0);
    else     n = min(n_wave0 + ni * 32 + (lane & 31), N - 1);
    w_rows[ni] = W + (size_t)n * K + (lane >> 5) * 32;
  }
  f32x16 acc[MT][NT];
#pragma unroll
  for (int mi = 0; mi < MT; ++mi)
#pragma unroll
    for (int ni = 0; ni < NT; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
  G::run(acc, x_rows, x_lds, w_rows, K / kBK, lds);

#pragma unroll
  for (int mi = 0; mi < MT; ++mi) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int m = m0 + mi * 32 + acc_row(lane, i);
      if (m >= M) continue;
      if (GLU) {
#pragma unroll
        for (int nj = 0; nj < NT / 2; ++nj) {
          const int n = n_wave0 + nj * 32 + acc_col(lane);
          if (n < N) ((bf16*)out)[(size_t)m * N + n] = (bf16)(silu_f(acc[mi][2 * nj][i]) * acc[mi][2 * nj + 1][i]);
        }
      } else {
#pragma unroll
        for (int ni = 0; ni < NT; ++ni) {
          const int n = n_wave0 + ni * 32 + acc_col(lane);
          if (n >= N) continue;
          const size_t o = (size_t)m * N + n;
          if (EPI == EPI_STORE) ((bf16*)out)[o] = (bf16)acc[mi][ni][i];
          else if (EPI == EPI_RESID_ADD) ((float*)out)[o] += acc[mi][ni][i];
          else ((float*)out)[o] = acc[mi][ni][i];
        }
      }
    }
  }
}

template <int MT, int NT, int EPI>
static void launch_mfma(const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const int32_t* a_rows,
                        const void* W, void* out, hipStream_t st) {
  using G = MfmaGemm<MT, NT, false>;
  constexpr int nout = (EPI == EPI_SWIGLU) ? 4 * NT * 16 : 4 * NT * 32;
  int m_blocks = (M_max + G::BM - 1) / G::BM, n_blocks = (N + nout - 1) / nout;
  int total = m_blocks * n_blocks;
  int grid = ((total + 7) / 8) * 8;
  hipLaunchKernelGGL((gemm_mfma_kernel<MT, NT, EPI>), dim3(grid), dim3(256), G::LDS_BYTES, st, n_rows_dev, M_max, N, K,
                     (const bf16*)A, a_rows, (const bf16*)W, out, m_blocks, n_blocks);
}

template <typename T, int EPI>
static void launch_simple(const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const int32_t* a_rows,
                          const void* W, void* out, hipStream_t st) {
  dim3 grid((N + 63) / 64, (M_max + 63) / 64);
  hipLaunchKernelGGL((gemm_simple_kernel<T, EPI>), grid, dim3(256), 0, st, n_rows_dev, M_max, N, K, (const T*)A, a_rows,
                     (const T*)W, out);
}

template <int EPI>
static void dispatch(int dtype, const int32_t* n_rows_dev, int M_max, int N, int K, const void* A,
                     const int32_t* a_rows, const void* W, void* out, hipStream_t st) {
  static const bool force_simple = getenv("BS_SIMPLE_GEMM") != nullptr;   // debugging aid
  if (dtype == BS_F32) { launch_simple<float, EPI>(n_rows_dev, M_max, N, K, A, a_rows, W, out, st); return; }
  if (force_simple) { launch_simple<bf16, EPI>(n_rows_dev, M_max, N, K, A, a_rows, W, out, st); return; }
  if (M_max <= 32) launch_mfma<1, 2, EPI>(n_rows_dev, M_max, N, K, A, a_rows, W, out, st);
  else if (M_max <= 64) launch_mfma<2, 2, EPI>(n_rows_dev, M_max, N, K, A, a_rows, W, out, st);
  else launch_mfma<4, 2, EPI>(n_rows_dev, M_max, N, K, A, a_rows, W, out, st);
}

void launch_gemm(int dtype, GemmEpilogue epi, const int32_t* n_rows_dev, int M_max, int N, int K, const void* A,
                 const int32_t* a_rows, const void* W, void* out, hipStream_t st) {
  switch (epi) {
    case EPI_STORE: dispatch<EPI_STORE>(dtype, n_rows_dev, M_max, N, K, A, a_rows, W, out, st); break;
    case EPI_RESID_ADD: dispatch<EPI_RESID_ADD>(dtype, n_rows_dev, M_max, N, K, A, a_rows, W, out, st); break;
    case EPI_SWIGLU: dispatch<EPI_SWIGLU>(dtype, n_rows_dev, M_max, N, K, A, a_rows, W, out, st); break;
    case EPI_STORE_F32: dispatch<EPI_STORE_F32>(dtype, n_rows_dev, M_max, N, K, A, a_rows, W, out, st); break;
  }
}
