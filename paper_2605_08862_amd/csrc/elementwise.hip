// Token-wise, bandwidth-trivial kernels of the verify pass (Sec. 3.3 "token-wise operations"):
// embedding gather, RMSNorm, rotary + tentative KV append, and the cache import/export copies.
// Each moves O(M*d) bytes per layer (<1 % of a step's traffic); they are written for clarity and
// coalesced row access, one workgroup per packed row.
#include "common.h"

template <typename T>
__global__ void __launch_bounds__(256) embed_kernel(Plan p, int d, const T* __restrict__ embed, float* __restrict__ h) {
  int r = blockIdx.x;
  if (r >= p.n_rows[0]) return;
  const T* src = embed + (size_t)p.row_tok[r] * d;
  float* dst = h + (size_t)r * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = to_f32<T>(src[i]);
}

__device__ __forceinline__ float block_sum_256(float v, float* red) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// out[r] = h[r] * gain / sqrt(mean(h[r]^2) + eps), float32 in; out is the GEMM operand type
// (float32 for float32 models, float16 for bf16 models).
// With n_slabs > 0 the row first absorbs the K-split slabs of the preceding residual projection:
// h[r] += sum_s slabs[s][r] (the updated residual is written back).
template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_kernel(Plan p, int d, float eps, float* __restrict__ h,
                                                      const float* __restrict__ slabs, int n_slabs, size_t slab_stride,
                                                      const float* __restrict__ gain, T* __restrict__ out) {
  __shared__ float red[4];
  int r = blockIdx.x;
  if (r >= p.n_rows[0]) return;
  float* x = h + (size_t)r * d;
  float ss = 0.f;
  typedef float f4 __attribute__((ext_vector_type(4)));
  if (n_slabs > 0) {                       // d is a multiple of 64: 16-byte accesses throughout
    const float* sl = slabs + (size_t)r * d;
    for (int i = threadIdx.x * 4; i < d; i += 1024) {
      f4 v = *(const f4*)(x + i);
      for (int s = 0; s < n_slabs; ++s) v += *(const f4*)(sl + (size_t)s * slab_stride + i);
      *(f4*)(x + i) = v;
      ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    }
  } else {
    for (int i = threadIdx.x * 4; i < d; i += 1024) {
      const f4 v = *(const f4*)(x + i);
      ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
    }
  }
  ss = block_sum_256(ss, red);
  float inv = 1.0f / sqrtf(ss / (float)d + eps);
  T* o = out + (size_t)r * d;
  for (int i = threadIdx.x; i < d; i += 256) o[i] = from_f32<T>(x[i] * inv * gain[i]);
}

// Rotary (pairs (j, j + D/2), angle = position * theta^(-2j/D)) on q and k of packed row r at
// absolute position c_b + i.  The QKV projection arrives in float32 (so each of q, k, v is rounded
// exactly once, after the rotation): q goes to the query buffer (float16 for bf16 models: it is an
// attention operand, not cache data), k and v to the slot's page in the cache dtype.  Angles are formed in float64: at positions
// of 3e4 a float32 angle is already off by ~2e-3 rad.
template <typename T, typename TQ, typename TP>
__global__ void __launch_bounds__(256) rope_append_kernel(Plan p, KvView kv, int Hq, int Hkv, int D, float theta,
                                                          const float* __restrict__ qkv, int n_slabs, size_t slab_stride,
                                                          TQ* __restrict__ q_out, TP* __restrict__ k_pages,
                                                          TP* __restrict__ v_pages) {
  __shared__ float s_cos[64], s_sin[64];
  int r = blockIdx.x;
  if (r >= p.n_rows[0]) return;
  const int b = p.row_seq[r];
  const int pos = p.seq_c[b] + p.row_pos[r];
  const int half = D / 2;
  if (threadIdx.x < half) {
    double inv = exp2(-2.0 * (double)threadIdx.x / (double)D * log2((double)theta));
    double sn, cs;
    sincos((double)pos * inv, &sn, &cs);
    s_cos[threadIdx.x] = (float)cs;
    s_sin[threadIdx.x] = (float)sn;
  }
  __syncthreads();
  const float* row = qkv + (size_t)r * (Hq + 2 * Hkv) * D;
  TQ* qrow = q_out + (size_t)r * Hq * D;
  const int page = kv.block_table[(size_t)p.seq_slot[b] * kv.max_pages + pos / kPage];
  const int tok = pos % kPage;
  const size_t pbase = (size_t)page * kv_page_elems(Hkv, D);
  // q heads and k heads: one thread per (head, pair)
  for (int idx = threadIdx.x; idx < (Hq + Hkv) * half; idx += blockDim.x) {
    int hh = idx / half, j = idx % half;
    const float* x = row + (size_t)hh * D;
    float x1 = x[j], x2 = x[j + half];
    for (int sl = 1; sl < n_slabs; ++sl) { x1 += x[sl * slab_stride + j]; x2 += x[sl * slab_stride + j + half]; }
    float c = s_cos[j], s = s_sin[j];
    float y1 = x1 * c - x2 * s, y2 = x2 * c + x1 * s;
    if (hh < Hq) {
      qrow[hh * D + j] = from_f32<TQ>(y1);
      qrow[hh * D + j + half] = from_f32<TQ>(y2);
    } else {
      int kh = hh - Hq;
      // rounded to the cache dtype T, stored in the page encoding TP
      k_pages[pbase + k_index<TP>(D, kh, tok, j)] = from_f32<TP>(to_f32<T>(from_f32<T>(y1)));
      k_pages[pbase + k_index<TP>(D, kh, tok, j + half)] = from_f32<TP>(to_f32<T>(from_f32<T>(y2)));
    }
  }
  const float* vrow = row + (size_t)(Hq + Hkv) * D;
  for (int idx = threadIdx.x; idx < Hkv * D; idx += blockDim.x) {
    int kh = idx / D, dd = idx % D;
    float v = vrow[idx];
    for (int sl = 1; sl < n_slabs; ++sl) v += vrow[sl * slab_stride + idx];
    v_pages[pbase + v_index<TP>(D, kh, tok, dd)] = from_f32<TP>(to_f32<T>(from_f32<T>(v)));
  }
}

template <typename T, typename TP>
__global__ void __launch_bounds__(256) kv_copy_kernel(KvView kv, int Hkv, int D, int slot, int pos0, TP* __restrict__ k_pages,
                                                      TP* __restrict__ v_pages, T* __restrict__ k_rows,
                                                      T* __restrict__ v_rows, int to_pages) {
  int i = blockIdx.x, pos = pos0 + i;
  int page = kv.block_table[(size_t)slot * kv.max_pages + pos / kPage];
  if (page < 0 || page >= kv.n_pages) return;
  int tok = pos % kPage;
  size_t pbase = (size_t)page * kv_page_elems(Hkv, D);
  for (int idx = threadIdx.x; idx < Hkv * D; idx += blockDim.x) {
    int kh = idx / D, dd = idx % D;
    size_t ki = pbase + k_index<TP>(D, kh, tok, dd), vi = pbase + v_index<TP>(D, kh, tok, dd);
    size_t ri = (size_t)i * Hkv * D + idx;
    if (to_pages) {
      k_pages[ki] = from_f32<TP>(to_f32<T>(k_rows[ri]));
      v_pages[vi] = from_f32<TP>(to_f32<T>(v_rows[ri]));
    } else {
      k_rows[ri] = from_f32<T>(to_f32<TP>(k_pages[ki]));
      v_rows[ri] = from_f32<T>(to_f32<TP>(v_pages[vi]));
    }
  }
}

void launch_embed(const Shape& s, const Plan& p, int M_max, const void* embed, float* h, hipStream_t st) {
  if (s.dtype == BS_F32) hipLaunchKernelGGL(embed_kernel<float>, dim3(M_max), dim3(256), 0, st, p, s.d, (const float*)embed, h);
  else hipLaunchKernelGGL(embed_kernel<bf16>, dim3(M_max), dim3(256), 0, st, p, s.d, (const bf16*)embed, h);
}
void launch_rmsnorm(const Shape& s, const Plan& p, int M_max, float* h, const float* slabs, int n_slabs,
                    const float* gain, void* out, hipStream_t st) {
  const size_t stride = (size_t)M_max * s.d;
  if (s.dtype == BS_F32)
    hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(M_max), dim3(256), 0, st, p, s.d, s.eps, h, slabs, n_slabs, stride, gain, (float*)out);
  else
    hipLaunchKernelGGL(rmsnorm_kernel<f16>, dim3(M_max), dim3(256), 0, st, p, s.d, s.eps, h, slabs, n_slabs, stride, gain, (f16*)out);
}
void launch_rope_append(const Shape& s, const Plan& p, const KvView& kv, int M_max, const float* qkv, int n_slabs,
                        void* q_out, void* k_pages, void* v_pages, hipStream_t st) {
  const size_t stride = (size_t)M_max * s.Nqkv();
  if (s.dtype == BS_F32)
    hipLaunchKernelGGL((rope_append_kernel<float, float, float>), dim3(M_max), dim3(256), 0, st, p, kv, s.Hq, s.Hkv, s.D, s.theta,
                       qkv, n_slabs, stride, (float*)q_out, (float*)k_pages, (float*)v_pages);
  else
    hipLaunchKernelGGL((rope_append_kernel<bf16, f16, f16>), dim3(M_max), dim3(256), 0, st, p, kv, s.Hq, s.Hkv, s.D, s.theta,
                       qkv, n_slabs, stride, (f16*)q_out, (f16*)k_pages, (f16*)v_pages);
}
void launch_kv_copy(const Shape& s, const KvView& kv, int slot, int pos0, int n, void* k_pages, void* v_pages,
                    void* k_rows, void* v_rows, bool to_pages, hipStream_t st) {
  if (n <= 0) return;
  if (s.dtype == BS_F32)
    hipLaunchKernelGGL((kv_copy_kernel<float, float>), dim3(n), dim3(256), 0, st, kv, s.Hkv, s.D, slot, pos0, (float*)k_pages,
                       (float*)v_pages, (float*)k_rows, (float*)v_rows, to_pages ? 1 : 0);
  else
    hipLaunchKernelGGL((kv_copy_kernel<bf16, f16>), dim3(n), dim3(256), 0, st, kv, s.Hkv, s.D, slot, pos0, (f16*)k_pages,
                       (f16*)v_pages, (bf16*)k_rows, (bf16*)v_rows, to_pages ? 1 : 0);
}
