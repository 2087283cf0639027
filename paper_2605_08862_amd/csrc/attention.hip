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
//     8-bit bf16 queries the logits of the 7B-shape slice drift by 3e-2).  The cache holds
//     bf16-rounded K/V values in float16 encoding, so page data are MFMA operands as they are.
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
}  // namespace

// NQ: query-row tiles (of 32) handled by one wave; QG: groups of waves, each group owning NQ of the
// workgroup's NQ*QG query tiles (tokens are split across the 4/QG waves of a group).
// Partial layout (n_split > 1): part_ml [B][Hkv][n_split][RP][2], part_o [B][Hkv][n_split][RP][D],
// RP = 32*NQ*QG.
template <int NQ, int QG, int D>
__global__ void __launch_bounds__(256) attn_mfma_kernel(Plan p, KvView kv, int Hq, int Hkv, float scale_log2e,
                                                        const f16* __restrict__ q, const f16* __restrict__ k_pages,
                                                        const f16* __restrict__ v_pages, f16* __restrict__ out,
                                                        float* __restrict__ part_o, float* __restrict__ part_ml,
                                                        int n_split) {
  constexpr int KS = D / 16;            // MFMA K-steps of the QK^T product
  constexpr int DT = D / 32;            // 32-wide d tiles of the output
  constexpr int RP = 32 * NQ * QG;      // padded query rows per workgroup
  constexpr int WPG = 4 / QG;           // waves per group (token split inside the workgroup)
  constexpr int SLOT = NQ * DT * 16 * 64;               // floats of one wave's output accumulator
  extern __shared__ __align__(16) char lds_raw[];
  float* s_o = (float*)lds_raw;                         // [2 slots][SLOT] accumulators in flight during the merge
  float* s_m = s_o + 2 * SLOT;                          // [4][32*NQ] per-wave running max
  float* s_l = s_m + 4 * 32 * NQ;                       // [4][32*NQ] per-wave sum

  const int h = blockIdx.x, b = blockIdx.y, split = blockIdx.z;
  const int k = p.seq_k[b];
  if (k < 0) return;
  const int G = Hq / Hkv;
  const int c = p.seq_c[b];
  const int n_tok = c + k + 1;
  const int R = (k + 1) * G;
  // the wave index is made scalar so that everything derived from it (tile index, block-table lookups)
  // stays on the scalar unit: a vector load of a page id inside the loop would force vmcnt(0) and
  // serialise the K/V prefetch
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int grp = wave / WPG, wig = wave % WPG;
  const int ln = lane & 31, lg = lane >> 5;
  const int row0 = p.row_start[b];
  const int32_t* bt = kv.block_table + (size_t)p.seq_slot[b] * kv.max_pages;
  const size_t page_elems = kv_page_elems(Hkv, D);

  // Query fragments (B operand: lane (n, g) holds Q[row n][g*D/2 + 8s + j]) are staged once in LDS in
  // fragment order and re-read per use: keeping them in registers would push the kernel into spills,
  // and a spill reload inside the loop forces vmcnt(0), i.e. it serialises the K/V prefetch.
  u32x4* s_q = (u32x4*)lds_raw;                         // [RP/32][KS][64] (aliases s_o; dead before the merge)
  int lim[NQ];                                          // last visible cache position of the lane's row
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    const int qr = (grp * NQ + qt) * 32 + ln;
    lim[qt] = (qr < R) ? c + qr / G : -1;
  }
  const int n_tiles = (n_tok + kTile - 1) / kTile;
  const int tps = (n_tiles + n_split - 1) / n_split;
  const int t_begin = split * tps, t_end = min(t_begin + tps, n_tiles);
  const bool group_active = (grp * NQ * 32) < R;        // wave-uniform
  auto load_tile = [&](int t, u32x4 (&kf)[KS], u32x4 (&vf)[DT * 2]) {
    const int tb = t * kTile;
    const int page = min(max(bt[tb / kPage], 0), kv.n_pages - 1);
    const size_t off = (size_t)page * page_elems + (size_t)(h * 2 + ((tb / kTile) & 1)) * (kTile * D) + lane * 8;
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[s] = *(const u32x4*)(k_pages + off + s * 512);
#pragma unroll
    for (int x = 0; x < DT * 2; ++x) vf[x] = *(const u32x4*)(v_pages + off + x * 512);
  };
  // register double buffering; the first tile is requested before the queries are staged so that its
  // latency overlaps that work
  u32x4 ka[KS], va[DT * 2], kb[KS], vb[DT * 2];
  int t = t_begin + wig;
  if (group_active && t < t_end) load_tile(t, ka, va);

  for (int f = wave; f < (RP / 32) * KS; f += 4) {      // one fragment (1 KiB) per wave iteration
    const int qtile = f / KS, s = f % KS;
    const int qr = qtile * 32 + ln;
    u32x4 v = u32x4{0, 0, 0, 0};
    if (qr < R) {
      const int iq = qr / G, hg = qr % G;
      v = *(const u32x4*)(q + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D + lg * (D / 2) + s * 8);
    }
    s_q[f * 64 + lane] = v;
  }
  __syncthreads();
  const u32x4* my_q = s_q + (size_t)(grp * NQ) * KS * 64 + lane;

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

  auto compute_tile = [&](int t, const u32x4 (&kc)[KS], const u32x4 (&vc)[DT * 2]) {
    const int tok0 = t * kTile + 16 * lg;               // accumulator register i <-> token tok0 + i
    const bool full = (t + 1) * kTile - 1 <= c;         // every token visible to every row: no masking
    f32x16 st[NQ];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
      for (int i = 0; i < 16; ++i) st[qt][i] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const f16x8 kh = as_f16x8(kc[s]);
#pragma unroll
      for (int qt = 0; qt < NQ; ++qt)
        st[qt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kh, as_f16x8(my_q[(qt * KS + s) * 64]), st[qt], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    f16x8 pf[NQ][2];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
      float x[16];
      if (full) {
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = st[qt][i];
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = (tok0 + i <= lim[qt]) ? st[qt][i] : -INFINITY;
      }
      float mloc = x[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mloc = fmaxf(mloc, x[i]);
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32)) * scale_log2e;       // scale > 0 commutes with max
      const float m_new = fmaxf(m_run[qt], mloc);
      const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_safe);
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        x[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], scale_log2e, -m_safe));   // exp2(-inf) = 0
        psum += x[i];
      }
      l_run[qt] = l_run[qt] * alpha + psum;             // per lane half; halves are added at the end
      m_run[qt] = m_new;
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[qt][dt][i] *= alpha;
      }
      pf[qt][0] = pack_f16x8(x);
      pf[qt][1] = pack_f16x8(x + 8);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
        const f16x8 vh = as_f16x8(vc[dt * 2 + t2]);
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt)
          o[qt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vh, pf[qt][t2], o[qt][dt], 0, 0, 0);
      }
  };

  if (group_active) {
    for (; t < t_end; t += WPG) {
      // current tile -> kb/vb (register moves), next tile requested into ka/va, then compute: the
      // loads of tile t+WPG are in flight during the whole computation of tile t
#pragma unroll
      for (int s = 0; s < KS; ++s) kb[s] = ka[s];
#pragma unroll
      for (int x = 0; x < DT * 2; ++x) vb[x] = va[x];
      load_tile(t + WPG < t_end ? t + WPG : t, ka, va);   // unconditional (the last one re-reads tile t): a
      compute_tile(t, kb, vb);                             // conditional prefetch costs vmcnt(0) waits
    }
  }
  __syncthreads();                                      // all waves are done with s_q before s_o reuses it

  // ---- merge the waves of each group (tree, accumulators cross LDS in register order) --------
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    l_run[qt] += __shfl_xor(l_run[qt], 32);
    if (lg == 0) {
      s_m[wave * 32 * NQ + qt * 32 + ln] = m_run[qt];
      s_l[wave * 32 * NQ + qt * 32 + ln] = l_run[qt];
    }
  }
  __syncthreads();
  float m_tot[NQ], l_tot[NQ];
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
    const float f_own = exp2f(m_run[qt] - ms);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[qt][dt][i] *= f_own;
  }
  // slot of a group: QG == 1 uses both slots in the first round, QG == 2 one slot per group
  auto put = [&](float* slot) {
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *(f32x4*)(slot + (((qt * DT + dt) * 4 + i4) * 64 + lane) * 4) =
              f32x4{o[qt][dt][4 * i4], o[qt][dt][4 * i4 + 1], o[qt][dt][4 * i4 + 2], o[qt][dt][4 * i4 + 3]};
  };
  auto add = [&](const float* slot) {
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const f32x4 v = *(const f32x4*)(slot + (((qt * DT + dt) * 4 + i4) * 64 + lane) * 4);
#pragma unroll
          for (int j = 0; j < 4; ++j) o[qt][dt][4 * i4 + j] += v[j];
        }
  };
  if (WPG == 4) {
    if (wig >= 2) put(s_o + (wig - 2) * SLOT);
    __syncthreads();
    if (wig < 2) add(s_o + wig * SLOT);
    __syncthreads();
    if (wig == 1) put(s_o);
    __syncthreads();
    if (wig == 0) add(s_o);
  } else {
    if (wig == 1) put(s_o + grp * SLOT);
    __syncthreads();
    if (wig == 0) add(s_o + grp * SLOT);
  }

  // ---- write from registers (first wave of each group): final rows or split partials -------------
  if (wig == 0) {
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
      const int qr = (grp * NQ + qt) * 32 + ln;
      if (qr >= R) continue;
      const int iq = qr / G, hg = qr % G;
      if (n_split == 1) {
        const float inv = 1.0f / l_tot[qt];
        f16* dst = out + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
            f16x4 v;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (f16)(o[qt][dt][4 * i4 + j] * inv);
            *(f16x4*)(dst + dt * 32 + 8 * i4 + 4 * lg) = v;
          }
      } else {
        const size_t pr = (((size_t)b * Hkv + h) * n_split + split) * RP + qr;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4)
            *(f32x4*)(part_o + pr * D + dt * 32 + 8 * i4 + 4 * lg) =
                f32x4{o[qt][dt][4 * i4], o[qt][dt][4 * i4 + 1], o[qt][dt][4 * i4 + 2], o[qt][dt][4 * i4 + 3]};
        if (lg == 0) { part_ml[pr * 2] = m_tot[qt]; part_ml[pr * 2 + 1] = l_tot[qt]; }
      }
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
  const size_t lds = (size_t)2 * NQ * (D / 32) * 16 * 64 * 4 + 2 * 4 * 32 * NQ * 4;   // two accumulator slots + statistics (>= the query fragments)
  float* part_ml = (float*)scratch;
  float* part_o = part_ml + (size_t)B * s.Hkv * n_split * RP * 2;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  auto kern = attn_mfma_kernel<NQ, QG, D>;
  static bool attr_set = false;
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr_set = true; }
  if (prof_token) attention_prof_mark(prof_token, st, true);
  hipLaunchKernelGGL(kern, dim3(s.Hkv, B, n_split), dim3(256), lds, st, p, kv, s.Hq, s.Hkv, scale_log2e,
                     (const f16*)q, (const f16*)k_pages, (const f16*)v_pages, (f16*)out, part_o, part_ml, n_split);
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
    hipLaunchKernelGGL((attn_simple_kernel<f16, f16>), dim3(M_max, s.Hq), dim3(256), 0, st, p, kv, s.Hq, s.Hkv, s.D, scale,
                       (const f16*)q, (const f16*)k_pages, (const f16*)v_pages, (f16*)out);
    return;
  }
  static const char* split_env = getenv("BS_ATTN_SPLIT");
  int n_split = split_env ? atoi(split_env) : (256 + B * s.Hkv / 2) / (B * s.Hkv);   // ~ one workgroup per CU
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
