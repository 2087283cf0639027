// Plain (non-MFMA) verify attention, any dtype / page layout: one workgroup per (packed row,
// query head).  Used by float32 models (the tiny parity configuration).  Sec. 3.3: every query
// length 1..k_max+1 is served by this one launch; row i of sequence b attends to cache
// positions 0 .. c_b + i (committed context plus the tentative rows up to itself).
#pragma once
#include "common.h"

template <typename T, typename TO>
__global__ void __launch_bounds__(256) attn_simple_kernel(Plan p, KvView kv, int Hq, int Hkv, int D, float scale,
                                                          const TO* __restrict__ q, const T* __restrict__ k_pages,
                                                          const T* __restrict__ v_pages, TO* __restrict__ out) {
  __shared__ float s_q[128], s_p[256], s_red[4], s_acc[2][128];
  const int r = blockIdx.x, hq = blockIdx.y;
  if (r >= p.n_rows[0]) return;
  const int b = p.row_seq[r];
  const int n_tok = p.seq_c[b] + p.row_pos[r] + 1;
  const int kvh = hq / (Hq / Hkv);
  const int tid = threadIdx.x;
  const int32_t* bt = kv.block_table + (size_t)p.seq_slot[b] * kv.max_pages;
  const size_t page_elems = kv_page_elems(Hkv, D);
  if (tid < D) s_q[tid] = to_f32<TO>(q[(size_t)r * Hq * D + (size_t)hq * D + tid]);
  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;      // acc: thread (tid%D, tid/D) partial of out[d]
  const int dd = tid % D, part = tid / D, nparts = 256 / D;
  __syncthreads();
  for (int t0 = 0; t0 < n_tok; t0 += 256) {
    const int t = t0 + tid;
    float s = -INFINITY;
    if (t < n_tok) {
      int page = min(max(bt[t / kPage], 0), kv.n_pages - 1);
      const T* kp = k_pages + (size_t)page * page_elems;
      float dot = 0.f;
      for (int d = 0; d < D; ++d) dot += s_q[d] * to_f32<T>(kp[k_index<T>(D, kvh, t % kPage, d)]);
      s = dot * scale;
    }
    float mx = s;
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) s_red[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    const float m_new = fmaxf(m_run, mx);
    const float pr = (t < n_tok) ? __expf(s - m_new) : 0.f;
    s_p[tid] = pr;
    float ps = pr;
    for (int o = 32; o > 0; o >>= 1) ps += __shfl_xor(ps, o);
    __syncthreads();                                   // s_red reads done, s_p visible
    if ((tid & 63) == 0) s_red[tid >> 6] = ps;
    __syncthreads();
    const float alpha = __expf(m_run - m_new);         // exp(-inf) = 0 on the first chunk
    l_run = l_run * alpha + (s_red[0] + s_red[1] + s_red[2] + s_red[3]);
    m_run = m_new;
    acc *= alpha;
    const int cnt = min(256, n_tok - t0);
    for (int j = part; j < cnt; j += nparts) {
      int tt = t0 + j;
      int page = min(max(bt[tt / kPage], 0), kv.n_pages - 1);
      acc += s_p[j] * to_f32<T>(v_pages[(size_t)page * page_elems + v_index<T>(D, kvh, tt % kPage, dd)]);
    }
    __syncthreads();
  }
  // combine the nparts partial sums per d
  if (part < 2) s_acc[part][dd] = 0.f;
  __syncthreads();
  for (int pp = 0; pp < nparts; ++pp) {
    if (part == pp) s_acc[0][dd] += acc;
    __syncthreads();
  }
  if (tid < D) out[(size_t)r * Hq * D + (size_t)hq * D + tid] = from_f32<TO>(s_acc[0][tid] / l_run);
}
