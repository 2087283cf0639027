// Token-wise, bandwidth-trivial kernels of the verify pass (Sec. 3.3 "token-wise operations"):
// embedding gather, RMSNorm, rotary + tentative KV append, and the cache import/export copies.
// Each moves O(M*d) bytes per layer (<1 % of a step's traffic); they are written for clarity and
// coalesced row access, one workgroup per packed row.
#include "common.h"
#include <type_traits>

// cos / sin of the rotary angle of packed row r (absolute position c_b + i) and pair j.  The angle is formed in
// float64 (at positions of 3e4 a float32 angle is already off by ~2e-3 rad), reduced to [-pi, pi] in float64 and
// only then handed to the float32 sine / cosine.
__device__ __forceinline__ void rope_angle(const Plan& p, int r, int j, int half, const double* __restrict__ inv_freq,
                                           float* __restrict__ cos_t, float* __restrict__ sin_t) {
  const int pos = p.seq_c[p.row_seq[r]] + p.row_pos[r];
  const double ang = (double)pos * inv_freq[j];
  const double two_pi_hi = 6.283185307179586, two_pi_lo = 2.4492935982947064e-16;
  const double n = rint(ang * 0.15915494309189535);
  const double red = fma(-n, two_pi_lo, fma(-n, two_pi_hi, ang));
  float sn, cs;
  sincosf((float)red, &sn, &cs);
  cos_t[(size_t)r * half + j] = cs;
  sin_t[(size_t)r * half + j] = sn;
}

// Token embedding of every packed row and, in the same launch, the row's rotary cos / sin table entries (the table
// [M_max][D/2] is shared by all layers of the step).
template <typename T>
__global__ void __launch_bounds__(256) embed_kernel(Plan p, int d, const T* __restrict__ embed, float* __restrict__ h,
                                                    int D, const double* __restrict__ inv_freq,
                                                    float* __restrict__ cos_t, float* __restrict__ sin_t) {
  int r = blockIdx.x;
  if (r >= p.n_rows[0]) return;
  const T* src = embed + (size_t)p.row_tok[r] * d;
  float* dst = h + (size_t)r * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = to_f32<T>(src[i]);
  if ((int)threadIdx.x < D / 2) rope_angle(p, r, threadIdx.x, D / 2, inv_freq, cos_t, sin_t);
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
// One workgroup per row; the row (d <= 1024 * NV floats) stays in registers between the sum of squares
// and the scaling, so every operand is read once and the kernel has a single barrier.
template <typename T> struct Vec4;
template <> struct Vec4<float> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct Vec4<f16> { typedef _Float16 type __attribute__((ext_vector_type(4))); };

template <typename T, int NV>
__global__ void __launch_bounds__(256) rmsnorm_kernel(Plan p, int d, float eps, float* __restrict__ h,
                                                      const float* __restrict__ slabs, SlabRule rule, size_t slab_stride,
                                                      const float* __restrict__ gain, T* __restrict__ out) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const int n_rows = p.n_rows[0];                        // a fixed slab count leaves this wait until the row's loads are in flight
  // With the device rule the slab count needs the row count before the first slab load anyway, so the rows beyond
  // the count leave here instead of loading what they never store (a step with 1185 of at most 2176 rows fetched
  // 123 MB per launch for 68 MB of live operands).
  if (rule.bm != 0 && r >= n_rows) return;
  const int n_slabs = rule.slabs(n_rows);
  typedef float f4 __attribute__((ext_vector_type(4)));
  float* x = h + (size_t)r * d;
  const float* sl = slabs + (size_t)r * d;
  f4 v[NV], gn[NV];
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    const int i = (it * 256 + threadIdx.x) * 4;          // d is a multiple of 64: 16-byte accesses throughout
    v[it] = f4{0.f, 0.f, 0.f, 0.f};
    gn[it] = v[it];
    if (i < d) {
      v[it] = *(const f4*)(x + i);
      gn[it] = *(const f4*)(gain + i);
    }
  }
  // slabs are added in index order; four slabs' loads are issued together (a slab index past the end is clamped
  // and its value dropped), so that a row costs one memory round trip instead of one per slab
  constexpr int GS = NV <= 4 ? 4 : 1;
  for (int s0 = 0; s0 < n_slabs; s0 += GS) {
    f4 t[GS][NV];
#pragma unroll
    for (int u = 0; u < GS; ++u) {
      const int s = min(s0 + u, n_slabs - 1);
#pragma unroll
      for (int it = 0; it < NV; ++it) {
        const int i = (it * 256 + threadIdx.x) * 4;
        t[u][it] = f4{0.f, 0.f, 0.f, 0.f};
        if (i < d) t[u][it] = *(const f4*)(sl + (size_t)s * slab_stride + i);
      }
    }
#pragma unroll
    for (int u = 0; u < GS; ++u)
      if (s0 + u < n_slabs) {
#pragma unroll
        for (int it = 0; it < NV; ++it) v[it] += t[u][it];
      }
  }
  if (r >= n_rows) return;                               // rows beyond the count: loaded (in bounds), never stored
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    const int i = (it * 256 + threadIdx.x) * 4;
    if (n_slabs > 0 && i < d) *(f4*)(x + i) = v[it];
    ss += v[it][0] * v[it][0] + v[it][1] * v[it][1] + v[it][2] * v[it][2] + v[it][3] * v[it][3];
  }
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = red[0] + red[1] + red[2] + red[3];
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  T* o = out + (size_t)r * d;
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    const int i = (it * 256 + threadIdx.x) * 4;
    if (i < d) {
      if constexpr (std::is_same<T, f16>::value) {
        *(f16x4*)(o + i) = to_f16x4_guarded(v[it][0] * inv * gn[it][0], v[it][1] * inv * gn[it][1],
                                            v[it][2] * inv * gn[it][2], v[it][3] * inv * gn[it][3], p.status);
      } else {
        typename Vec4<T>::type w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = from_f32<T>(v[it][e] * inv * gn[it][e]);
        *(typename Vec4<T>::type*)(o + i) = w;
      }
    }
  }
}

// Inverse rotary frequencies theta^(-2j/D), j < D/2, in float64 (filled once per context).
__global__ void rope_table_kernel(int D, float theta, double* __restrict__ inv_freq) {
  const int j = threadIdx.x;
  if (j < D / 2) inv_freq[j] = exp2(-2.0 * (double)j / (double)D * log2((double)theta));
}

// Rotary (pairs (j, j + D/2), angle = position * theta^(-2j/D)) on q and k of packed row r at
// absolute position c_b + i, with the cos / sin table filled by embed_kernel.  The QKV projection arrives in
// float32, as n_slabs K-split slabs that are summed here (so each of q, k, v is rounded exactly once, after
// the rotation): q goes to the query buffer (float16 for bf16 models: it is an attention operand, not
// cache data), k and v to the slot's page in the cache dtype.
// One workgroup per row; a work item is four consecutive rotation pairs of one head (two 16-byte loads
// per slab, 8-byte stores) or four consecutive v elements.
template <typename T, typename TQ, typename TP>
__global__ void __launch_bounds__(256) rope_append_kernel(Plan p, KvView kv, int Hq, int Hkv, int D,
                                                          const float* __restrict__ cos_t, const float* __restrict__ sin_t,
                                                          const float* __restrict__ qkv, int n_slabs, size_t slab_stride,
                                                          TQ* __restrict__ q_out, TP* __restrict__ k_pages,
                                                          TP* __restrict__ v_pages) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const int r = blockIdx.x;
  if (r >= p.n_rows[0]) return;
  const int b = p.row_seq[r];
  const int pos = p.seq_c[b] + p.row_pos[r];
  const int half = D / 2, groups = half / 4;
  const float* row = qkv + (size_t)r * (Hq + 2 * Hkv) * D;
  const int n_rot = (Hq + Hkv) * groups, n_items = n_rot + Hkv * D / 4;
  TQ* qrow = q_out + (size_t)r * Hq * D;
  const int page = kv.block_table[(size_t)p.seq_slot[b] * kv.max_pages + pos / kPage];
  const int tok = pos % kPage;
  const size_t pbase = (size_t)page * kv_page_elems(Hkv, D);
  for (int idx = threadIdx.x; idx < n_items; idx += 256) {
    if (idx < n_rot) {
      const int hh = idx / groups, j = (idx % groups) * 4;
      const float* x = row + (size_t)hh * D + j;
      f4 x1 = f4{0.f, 0.f, 0.f, 0.f}, x2 = x1;
      for (int sl = 0; sl < n_slabs; ++sl) { x1 += *(const f4*)(x + sl * slab_stride); x2 += *(const f4*)(x + sl * slab_stride + half); }
      const f4 c = *(const f4*)(cos_t + (size_t)r * half + j), sn = *(const f4*)(sin_t + (size_t)r * half + j);
      float y1[4], y2[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        y1[e] = x1[e] * c[e] - x2[e] * sn[e];
        y2[e] = x2[e] * c[e] + x1[e] * sn[e];
      }
      if (hh < Hq) {
        if constexpr (std::is_same<TQ, f16>::value) {
          *(f16x4*)(qrow + hh * D + j) = to_f16x4_guarded(y1[0], y1[1], y1[2], y1[3], p.status);
          *(f16x4*)(qrow + hh * D + j + half) = to_f16x4_guarded(y2[0], y2[1], y2[2], y2[3], p.status);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            qrow[hh * D + j + e] = from_f32<TQ>(y1[e]);
            qrow[hh * D + j + half + e] = from_f32<TQ>(y2[e]);
          }
        }
      } else {
        const int kh = hh - Hq;
        // rounded to the cache dtype T, stored in the page encoding TP (four consecutive d are contiguous in
        // both page layouts)
        TP* k1 = k_pages + pbase + k_index<TP>(D, kh, tok, j);
        TP* k2 = k_pages + pbase + k_index<TP>(D, kh, tok, j + half);
        if constexpr (std::is_same<TP, f16>::value) {
          auto rt = [](float x) { return to_f32<T>(from_f32<T>(x)); };
          *(f16x4*)k1 = to_f16x4_guarded(rt(y1[0]), rt(y1[1]), rt(y1[2]), rt(y1[3]), p.status);
          *(f16x4*)k2 = to_f16x4_guarded(rt(y2[0]), rt(y2[1]), rt(y2[2]), rt(y2[3]), p.status);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            k1[e] = from_f32<TP>(to_f32<T>(from_f32<T>(y1[e])));
            k2[e] = from_f32<TP>(to_f32<T>(from_f32<T>(y2[e])));
          }
        }
      }
    } else {
      const int e0 = (idx - n_rot) * 4;                  // four consecutive v elements of one head
      const int kh = e0 / D, dd = e0 % D;
      const float* x = row + (size_t)(Hq + Hkv) * D + e0;
      f4 v = f4{0.f, 0.f, 0.f, 0.f};
      for (int sl = 0; sl < n_slabs; ++sl) v += *(const f4*)(x + sl * slab_stride);
      if constexpr (std::is_same<TP, f16>::value) {
        auto rt = [](float x) { return to_f32<T>(from_f32<T>(x)); };
        const f16x4 w = to_f16x4_guarded(rt(v[0]), rt(v[1]), rt(v[2]), rt(v[3]), p.status);
#pragma unroll
        for (int e = 0; e < 4; ++e) v_pages[pbase + v_index<TP>(D, kh, tok, dd + e)] = w[e];
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          v_pages[pbase + v_index<TP>(D, kh, tok, dd + e)] = from_f32<TP>(to_f32<T>(from_f32<T>(v[e])));
      }
    }
  }
}

template <typename T, typename TP>
__global__ void __launch_bounds__(256) kv_copy_kernel(KvView kv, int Hkv, int D, int slot, int pos0, TP* __restrict__ k_pages,
                                                      TP* __restrict__ v_pages, T* __restrict__ k_rows,
                                                      T* __restrict__ v_rows, int to_pages, int32_t* __restrict__ status) {
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
      float kx = to_f32<T>(k_rows[ri]), vx = to_f32<T>(v_rows[ri]);
      if constexpr (std::is_same<TP, f16>::value) {      // imported bf16 values beyond the float16 range
        if (!(fabsf(kx) <= 65504.f) || !(fabsf(vx) <= 65504.f)) {
          kx = f16_saturate(kx); vx = f16_saturate(vx);
          atomicOr(status, BS_FAULT_RANGE);
        }
      }
      k_pages[ki] = from_f32<TP>(kx);
      v_pages[vi] = from_f32<TP>(vx);
    } else {
      k_rows[ri] = from_f32<T>(to_f32<TP>(k_pages[ki]));
      v_rows[ri] = from_f32<T>(to_f32<TP>(v_pages[vi]));
    }
  }
}

void launch_embed(const Shape& s, const Plan& p, int M_max, const void* embed, float* h, const double* inv_freq,
                  float* cos_t, float* sin_t, hipStream_t st) {
  if (s.dtype == BS_F32)
    hipLaunchKernelGGL(embed_kernel<float>, dim3(M_max), dim3(256), 0, st, p, s.d, (const float*)embed, h, s.D, inv_freq, cos_t, sin_t);
  else
    hipLaunchKernelGGL(embed_kernel<bf16>, dim3(M_max), dim3(256), 0, st, p, s.d, (const bf16*)embed, h, s.D, inv_freq, cos_t, sin_t);
}
void launch_rmsnorm(const Shape& s, const Plan& p, int M_max, float* h, const float* slabs, const SlabRule& n_slabs,
                    const float* gain, void* out, hipStream_t st) {
  const size_t stride = (size_t)M_max * s.d;
#define BS_RMS(T_, NV_) hipLaunchKernelGGL((rmsnorm_kernel<T_, NV_>), dim3(M_max), dim3(256), 0, st, p, s.d, s.eps, h, slabs, n_slabs, stride, gain, (T_*)out)
  if (s.dtype == BS_F32) { if (s.d <= 2048) BS_RMS(float, 2); else if (s.d <= 4096) BS_RMS(float, 4); else BS_RMS(float, 16); }
  else                   { if (s.d <= 2048) BS_RMS(f16, 2);   else if (s.d <= 4096) BS_RMS(f16, 4);   else BS_RMS(f16, 16); }
#undef BS_RMS
}
void launch_rope_table(const Shape& s, double* inv_freq, hipStream_t st) {
  hipLaunchKernelGGL(rope_table_kernel, dim3(1), dim3(64), 0, st, s.D, s.theta, inv_freq);
}
void launch_rope_append(const Shape& s, const Plan& p, const KvView& kv, int M_max, const float* cos_t, const float* sin_t,
                        const float* qkv, int n_slabs, void* q_out, void* k_pages, void* v_pages, hipStream_t st) {
  const size_t stride = (size_t)M_max * s.Nqkv();
  if (s.dtype == BS_F32)
    hipLaunchKernelGGL((rope_append_kernel<float, float, float>), dim3(M_max), dim3(256), 0, st, p, kv, s.Hq, s.Hkv, s.D, cos_t, sin_t,
                       qkv, n_slabs, stride, (float*)q_out, (float*)k_pages, (float*)v_pages);
  else
    hipLaunchKernelGGL((rope_append_kernel<bf16, f16, f16>), dim3(M_max), dim3(256), 0, st, p, kv, s.Hq, s.Hkv, s.D, cos_t, sin_t,
                       qkv, n_slabs, stride, (f16*)q_out, (f16*)k_pages, (f16*)v_pages);
}
void launch_kv_copy(const Shape& s, const KvView& kv, int slot, int pos0, int n, void* k_pages, void* v_pages,
                    void* k_rows, void* v_rows, bool to_pages, int32_t* status, hipStream_t st) {
  if (n <= 0) return;
  if (s.dtype == BS_F32)
    hipLaunchKernelGGL((kv_copy_kernel<float, float>), dim3(n), dim3(256), 0, st, kv, s.Hkv, s.D, slot, pos0, (float*)k_pages,
                       (float*)v_pages, (float*)k_rows, (float*)v_rows, to_pages ? 1 : 0, status);
  else
    hipLaunchKernelGGL((kv_copy_kernel<bf16, f16>), dim3(n), dim3(256), 0, st, kv, s.Hkv, s.D, slot, pos0, (f16*)k_pages,
                       (f16*)v_pages, (bf16*)k_rows, (bf16*)v_rows, to_pages ? 1 : 0, status);
}
