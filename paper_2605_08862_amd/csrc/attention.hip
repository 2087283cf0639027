// Ragged multi-query verify attention (Sec. 3.3 "unified attention"): one launch serves every
// sequence of the batch whatever its number of query positions (1 .. k_max+1); query row i of
// sequence b attends to cache positions 0 .. c_b + i.
//
// MI355X design (bf16 models).  The kernel is HBM-bound: it must stream the committed K/V once.
//   * A workgroup owns (sequence, KV head, KV split).  All (k_b+1)*G query rows that share the KV
//     head are packed into 32-row MFMA tiles, so K/V are read once for all of them (the paper's
//     point: the extra draft rows ride in the matrix tile for free).
//   * The 4 waves of a workgroup take different 32-token tiles; each keeps its own online-softmax
//     state (running max m, sum l) and output accumulator and they are merged once at the end.
//   * K/V pages are stored in MFMA operand order (see common.h), so a wave's 16-byte-per-lane
//     load is one contiguous 1 KiB read that lands directly in the operand registers: no LDS
//     staging, no bank conflicts, no shuffles.  LDS is used only for the final cross-wave merge.
//   * Arithmetic runs on the f16 MFMA: queries and probabilities carry 11 significant bits (with
//     8-bit bf16 queries the logits of the 7B-shape slice drift by 3e-2); the bf16 K/V fragments are
//     widened to float16 in registers (exact for 6.1e-5 <= |x| <= 65504) right before use.
//   * S^T = K Q^T (tokens are accumulator rows, the lane is the query row), so the softmax
//     statistics of a query row are lane-private apart from one exchange between the two lane
//     halves, and the probabilities are already laid out as the B operand of O^T = V^T P^T.
// float32 models use the plain kernel in attn_simple.h.
#include "attn_simple.h"
#include "gemm_mfma.h"
#include <stdlib.h>

namespace {
constexpr int kMaxSplit = 16;

__device__ __forceinline__ f16x8 pack_f16x8(const float* v) {
  f16x8 r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r[j] = (f16)v[j];
  return r;
}
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
// eight bf16 (packed in four dwords) -> eight float16; three VALU ops per pair
__device__ __forceinline__ f16x8 widen_bf16x8(u32x4 v) {
  f16x8 r;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = __uint_as_float(v[j] << 16), hi = __uint_as_float(v[j] & 0xffff0000u);
    const f16x2 pr = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(lo, hi));   // exact: no rounding occurs
    r[2 * j] = pr[0];
    r[2 * j + 1] = pr[1];
  }
  return r;
}
}  // namespace

// NQ: query-row tiles (of 32) handled by one wave; QG: groups of waves, each group owning NQ of the
// workgroup's NQ*QG query tiles (tokens are split across the 4/QG waves of a group).
// Partial layout (n_split > 1): part_ml [B][Hkv][n_split][RP][2], part_o [B][Hkv][n_split][RP][D],
// RP = 32*NQ*QG.
template <int NQ, int QG, int D>
__global__ void __launch_bounds__(256) attn_mfma_kernel(Plan p, KvView kv, int Hq, int Hkv, float scale_log2e,
                                                        const f16* __restrict__ q, const bf16* __restrict__ k_pages,
                                                        const bf16* __restrict__ v_pages, f16* __restrict__ out,
                                                        float* __restrict__ part_o, float* __restrict__ part_ml,
                                                        int n_split) {
  constexpr int KS = D / 16;            // MFMA K-steps of the QK^T product
  constexpr int DT = D / 32;            // 32-wide d tiles of the output
  constexpr int RP = 32 * NQ * QG;      // padded query rows per workgroup
  constexpr int WPG = 4 / QG;           // waves per group (token split inside the workgroup)
  constexpr int DS = D + 4;             // LDS row stride of the merged accumulator (bank spread)
  extern __shared__ __align__(16) char lds_raw[];
  float* s_o = (float*)lds_raw;                         // [RP][DS] merged output accumulator
  float* s_m = s_o + RP * DS;                           // [4][32*NQ] per-wave running max
  float* s_l = s_m + 4 * 32 * NQ;                       // [4][32*NQ] per-wave sum

  const int h = blockIdx.x, b = blockIdx.y, split = blockIdx.z;
  const int k = p.seq_k[b];
  if (k < 0) return;
  const int G = Hq / Hkv;
  const int c = p.seq_c[b];
  const int n_tok = c + k + 1;
  const int R = (k + 1) * G;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int grp = wave / WPG, wig = wave % WPG;
  const int ln = lane & 31, lg = lane >> 5;
  const int row0 = p.row_start[b];
  const int32_t* bt = kv.block_table + (size_t)p.seq_slot[b] * kv.max_pages;
  const size_t page_elems = kv_page_elems(Hkv, D);

  // query fragments (B operand): lane (n, g) holds Q[row n][g*D/2 + 8s + j]
  u32x4 qf[NQ][KS];
  int lim[NQ];                                          // last visible cache position of the lane's row
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    const int qr = (grp * NQ + qt) * 32 + ln;
    if (qr < R) {
      const int iq = qr / G, hg = qr % G;
      const f16* qp = q + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D + lg * (D / 2);
#pragma unroll
      for (int s = 0; s < KS; ++s) qf[qt][s] = *(const u32x4*)(qp + s * 8);
      lim[qt] = c + iq;
    } else {
#pragma unroll
      for (int s = 0; s < KS; ++s) qf[qt][s] = u32x4{0, 0, 0, 0};
      lim[qt] = -1;
    }
  }
  f32x16 o[NQ][DT];
  float m_run[NQ], l_run[NQ];
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[qt][dt][i] = 0.f;
  }

  const int n_tiles = (n_tok + kTile - 1) / kTile;
  const int tps = (n_tiles + n_split - 1) / n_split;
  const int t_begin = split * tps, t_end = min(t_begin + tps, n_tiles);
  const bool group_active = (grp * NQ * 32) < R;        // wave-uniform

  auto tile_ptrs = [&](int t, const bf16*& kp, const bf16*& vp) {
    const int tb = t * kTile;
    const int page = min(max(bt[tb / kPage], 0), kv.n_pages - 1);
    const size_t off = (size_t)page * page_elems + (size_t)(h * 2 + ((tb / kTile) & 1)) * (kTile * D) + lane * 8;
    kp = k_pages + off;
    vp = v_pages + off;
  };

  if (group_active) {
    u32x4 kf[KS], vf[DT * 2];
    int t = t_begin + wig;
    if (t < t_end) {
      const bf16 *kp, *vp;
      tile_ptrs(t, kp, vp);
#pragma unroll
      for (int s = 0; s < KS; ++s) kf[s] = *(const u32x4*)(kp + s * 512);
#pragma unroll
      for (int x = 0; x < DT * 2; ++x) vf[x] = *(const u32x4*)(vp + x * 512);
    }
    for (; t < t_end; t += WPG) {
      u32x4 kc[KS], vc[DT * 2];
#pragma unroll
      for (int s = 0; s < KS; ++s) kc[s] = kf[s];
#pragma unroll
      for (int x = 0; x < DT * 2; ++x) vc[x] = vf[x];
      if (t + WPG < t_end) {                            // prefetch the wave's next tile
        const bf16 *kp, *vp;
        tile_ptrs(t + WPG, kp, vp);
#pragma unroll
        for (int s = 0; s < KS; ++s) kf[s] = *(const u32x4*)(kp + s * 512);
#pragma unroll
        for (int x = 0; x < DT * 2; ++x) vf[x] = *(const u32x4*)(vp + x * 512);
      }
      const int tok0 = t * kTile + 16 * lg;             // accumulator register i <-> token tok0 + i
      f32x16 st[NQ];
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i) st[qt][i] = 0.f;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const f16x8 kh = widen_bf16x8(kc[s]);
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt)
          st[qt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kh, as_f16x8(qf[qt][s]), st[qt], 0, 0, 0);
      }
      f16x8 pf[NQ][2];
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt) {
        float x[16];
        float mloc = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          x[i] = (tok0 + i <= lim[qt]) ? st[qt][i] * scale_log2e : -INFINITY;
          mloc = fmaxf(mloc, x[i]);
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float m_new = fmaxf(m_run[qt], mloc);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f(m_run[qt] - m_safe);
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) { x[i] = exp2f(x[i] - m_safe); psum += x[i]; }
        l_run[qt] = l_run[qt] * alpha + psum;           // per lane half; halves are added at the end
        m_run[qt] = m_new;
        if (__any(alpha != 1.0f)) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[qt][dt][i] *= alpha;
        }
        pf[qt][0] = pack_f16x8(x);
        pf[qt][1] = pack_f16x8(x + 8);
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          const f16x8 vh = widen_bf16x8(vc[dt * 2 + t2]);
#pragma unroll
          for (int qt = 0; qt < NQ; ++qt)
            o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vh, pf[qt][t2], o[qt][dt], 0, 0, 0);
        }
    }
  }

  // ---- merge the waves of each group -------------------------------------------------------
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    l_run[qt] += __shfl_xor(l_run[qt], 32);
    if (lg == 0) {
      s_m[wave * 32 * NQ + qt * 32 + ln] = m_run[qt];
      s_l[wave * 32 * NQ + qt * 32 + ln] = l_run[qt];
    }
  }
  __syncthreads();
  float m_tot[NQ], l_tot[NQ], f_own[NQ];
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    float mt = -INFINITY;
#pragma unroll
    for (int w = 0; w < WPG; ++w) mt = fmaxf(mt, s_m[(grp * WPG + w) * 32 * NQ + qt * 32 + ln]);
    const float ms = (mt == -INFINITY) ? 0.f : mt;
    float lt = 0.f;
#pragma unroll
    for (int w = 0; w < WPG; ++w) {
      const int o2 = (grp * WPG + w) * 32 * NQ + qt * 32 + ln;
      lt += s_l[o2] * exp2f(s_m[o2] - ms);
    }
    m_tot[qt] = mt;
    l_tot[qt] = lt;
    f_own[qt] = exp2f(m_run[qt] - ms);
  }
  for (int w = 0; w < WPG; ++w) {                       // deterministic order: wave 0 stores, others add
    if (wig == w) {
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt) {
        float* dst = s_o + (size_t)((grp * NQ + qt) * 32 + ln) * DS;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int d = dt * 32 + acc_row(lane, i);
            const float v = o[qt][dt][i] * f_own[qt];
            if (w == 0) dst[d] = v; else dst[d] += v;
          }
      }
    }
    __syncthreads();
  }
  if (wig == 0 && lg == 0) {                            // publish the group's totals for the writers
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
      s_m[(grp * WPG) * 32 * NQ + qt * 32 + ln] = m_tot[qt];
      s_l[(grp * WPG) * 32 * NQ + qt * 32 + ln] = l_tot[qt];
    }
  }
  __syncthreads();

  // ---- write: final rows (n_split == 1) or partials ------------------------------------------
  for (int idx = threadIdx.x; idx < RP * (D / 4); idx += 256) {
    const int qr = idx / (D / 4), d4 = (idx % (D / 4)) * 4;
    if (qr >= R) continue;
    const int g2 = qr / (32 * NQ), qt = (qr / 32) % NQ, n = qr % 32;
    const float mt = s_m[(g2 * WPG) * 32 * NQ + qt * 32 + n], lt = s_l[(g2 * WPG) * 32 * NQ + qt * 32 + n];
    const float* src = s_o + (size_t)qr * DS + d4;
    if (n_split == 1) {
      const int iq = qr / G, hg = qr % G;
      const float inv = 1.0f / lt;
      f16* dst = out + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D + d4;
#pragma unroll
      for (int j = 0; j < 4; ++j) dst[j] = (f16)(src[j] * inv);
    } else {
      const size_t pr = (((size_t)b * Hkv + h) * n_split + split) * RP + qr;
      *(f32x4*)(part_o + pr * D + d4) = *(const f32x4*)src;
      if (d4 == 0) { part_ml[pr * 2] = mt; part_ml[pr * 2 + 1] = lt; }
    }
  }
}

// Combines the KV splits of one (packed row, query head): standard log-sum-exp merge.
template <int D>
__global__ void __launch_bounds__(D) attn_merge_kernel(Plan p, int Hq, int Hkv, int RP, const float* __restrict__ part_o,
                                                       const float* __restrict__ part_ml, int n_split,
                                                       f16* __restrict__ out) {
  const int r = blockIdx.x, hq = blockIdx.y;
  if (r >= p.n_rows[0]) return;
  const int b = p.row_seq[r], iq = p.row_pos[r];
  const int G = Hq / Hkv, h = hq / G, hg = hq % G;
  const int qr = iq * G + hg;
  const size_t base = (((size_t)b * Hkv + h) * n_split) * RP + qr;
  float mt = -INFINITY;
  for (int s = 0; s < n_split; ++s) mt = fmaxf(mt, part_ml[(base + (size_t)s * RP) * 2]);
  float lt = 0.f, acc = 0.f;
  for (int s = 0; s < n_split; ++s) {
    const size_t pr = base + (size_t)s * RP;
    const float m = part_ml[pr * 2];
    if (m == -INFINITY) continue;
    const float f = exp2f(m - mt);
    lt += part_ml[pr * 2 + 1] * f;
    acc += part_o[pr * D + threadIdx.x] * f;
  }
  out[(size_t)r * Hq * D + (size_t)hq * D + threadIdx.x] = (f16)(acc / lt);
}

static int rows_padded(const Shape& s, int k_max) {
  int R = (k_max + 1) * (s.Hq / s.Hkv);
  int tiles = (R + 31) / 32;
  if (tiles <= 2) return tiles * 32;
  return 128;
}

size_t attention_scratch_bytes(const Shape& s, int B_max, int k_max) {
  if (s.dtype != BS_BF16) return 256;
  size_t rp = rows_padded(s, k_max);
  return (size_t)B_max * s.Hkv * kMaxSplit * rp * (s.D + 2) * sizeof(float);
}

template <int NQ, int QG, int D>
static void launch_mfma_attn(const Shape& s, const Plan& p, const KvView& kv, int B, int M_max, const void* q,
                             const void* k_pages, const void* v_pages, void* out, void* scratch, int n_split,
                             void* prof_token, hipStream_t st) {
  constexpr int RP = 32 * NQ * QG;
  const size_t lds = (size_t)RP * (D + 4) * 4 + 2 * 4 * 32 * NQ * 4;
  float* part_ml = (float*)scratch;
  float* part_o = part_ml + (size_t)B * s.Hkv * n_split * RP * 2;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  auto kern = attn_mfma_kernel<NQ, QG, D>;
  static bool attr_set = false;
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr_set = true; }
  if (prof_token) attention_prof_mark(prof_token, st, true);
  hipLaunchKernelGGL(kern, dim3(s.Hkv, B, n_split), dim3(256), lds, st, p, kv, s.Hq, s.Hkv, scale_log2e,
                     (const f16*)q, (const bf16*)k_pages, (const bf16*)v_pages, (f16*)out, part_o, part_ml, n_split);
  if (prof_token) attention_prof_mark(prof_token, st, false);
  if (n_split > 1)
    hipLaunchKernelGGL(attn_merge_kernel<D>, dim3(M_max, s.Hq), dim3(D), 0, st, p, s.Hq, s.Hkv, RP, part_o, part_ml,
                       n_split, (f16*)out);
}

void launch_attention(const Shape& s, const Plan& p, const KvView& kv, int B, int k_max, int M_max, const void* q,
                      const void* k_pages, const void* v_pages, void* out, void* scratch, void* prof_token,
                      hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)s.D);
  static const bool force_simple = getenv("BS_SIMPLE_ATTN") != nullptr;   // debugging aid
  if (s.dtype == BS_F32) {
    hipLaunchKernelGGL((attn_simple_kernel<float, float>), dim3(M_max, s.Hq), dim3(256), 0, st, p, kv, s.Hq, s.Hkv, s.D, scale,
                       (const float*)q, (const float*)k_pages, (const float*)v_pages, (float*)out);
    return;
  }
  if (force_simple) {
    hipLaunchKernelGGL((attn_simple_kernel<bf16, f16>), dim3(M_max, s.Hq), dim3(256), 0, st, p, kv, s.Hq, s.Hkv, s.D, scale,
                       (const f16*)q, (const bf16*)k_pages, (const bf16*)v_pages, (f16*)out);
    return;
  }
  static const char* split_env = getenv("BS_ATTN_SPLIT");
  int n_split = split_env ? atoi(split_env) : (1024 + B * s.Hkv - 1) / (B * s.Hkv);
  n_split = n_split < 1 ? 1 : (n_split > kMaxSplit ? kMaxSplit : n_split);
  const int tiles = (rows_padded(s, k_max)) / 32;
#define BS_ATTN(NQ, QG)                                                                                         \
  do {                                                                                                          \
    if (s.D == 128) launch_mfma_attn<NQ, QG, 128>(s, p, kv, B, M_max, q, k_pages, v_pages, out, scratch, n_split, prof_token, st); \
    else launch_mfma_attn<NQ, QG, 64>(s, p, kv, B, M_max, q, k_pages, v_pages, out, scratch, n_split, prof_token, st);   \
  } while (0)
  if (tiles == 1) BS_ATTN(1, 1);
  else if (tiles == 2) BS_ATTN(2, 1);
  else BS_ATTN(2, 2);
#undef BS_ATTN
}
