// Ragged multi-query verify attention (Sec. 3.3 "unified attention"): one launch serves every
// sequence of the batch whatever its number of query positions (1 .. k_max+1); query row i of
// sequence b attends to cache positions 0 .. c_b + i.
//
// MI355X design (bf16 models).  The kernel is HBM-bound: it must stream the committed K/V once.
//   * A workgroup owns (sequence, KV head, token chunk, query block).  All (k_b+1)*G query rows that
//     share the KV head are packed into 32-row MFMA tiles, so K/V are read from HBM once for all of
//     them (the paper's point: the extra draft rows ride in the matrix tile for free).  When there
//     are too few (sequence, KV head) units for 256 CUs, the query tiles of a unit go to different
//     workgroups placed on one XCD (shared L2) rather than splitting the token range: no partial
//     results (measured, batch 64 x 2 KV heads, context 2048: 31 us against 35 us + a 6.6 us merge
//     kernel for a two-way token split).
//   * Token chunks come from the step's work list (plan_kernel): one common chunk size for the whole
//     batch, so a 32768-token sequence next to 512-token ones becomes many equal work items instead of
//     one workgroup that runs 60 times longer than the others.  A sequence with one chunk writes its
//     rows directly; with several, every workgroup stores a float32 partial (+ max, sum) and the LAST
//     one to finish (device-scope counter, no waiting anywhere) merges them.
//   * The 4 waves of a workgroup take different 32-token tiles; each keeps its own online-softmax
//     state (running max m, sum l) and output accumulator and they are merged once at the end.
//   * K/V pages are stored in MFMA operand order (see common.h), so a wave's 16-byte-per-lane
//     load is one contiguous 1 KiB read that lands directly in the operand registers: no LDS
//     staging, no bank conflicts, no shuffles.  LDS holds the query fragments and, at the end, the cross-wave merge.
//   * Arithmetic runs on the f16 MFMA: queries and probabilities carry 11 significant bits (with
//     8-bit bf16 queries the logits of the 7B-shape slice drift by 3e-2).  The cache holds
//     bf16-rounded K/V values in float16 encoding, so page data are MFMA operands as they are.
//   * S^T = K Q^T (tokens are accumulator rows, the lane is the query row), so the softmax
//     statistics of a query row are lane-private apart from one exchange between the two lane
//     halves, and the probabilities are already laid out as the B operand of O^T = V^T P^T.
// float32 models use the plain kernel in attn_simple.h.
#include "attn_simple.h"
#include "attn_wide.h"
#include "gemm_mfma.h"
#include <type_traits>

namespace {

__device__ __forceinline__ f16x8 pack_f16x8(const float* v) {
  f16x8 r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r[j] = (f16)v[j];
  return r;
}
}  // namespace

// NQ: query-row tiles (of 32) handled by one wave; QG: groups of waves, each group owning NQ of the
// workgroup's NQ*QG query tiles (tokens are split across the 4/QG waves of a group).
// A unit = (work item, KV head) is covered by q_blocks workgroups (NQ*QG query tiles each).  Workgroups of
// different query blocks stream the same K/V; the one-dimensional grid is decoded so that all workgroups of a
// unit run on the same XCD (ids are dealt round-robin to the 8 XCDs) and are dispatched back to back, so the
// second reader hits that XCD's L2 and HBM is still read once.
// Partials (sequences with several chunks): part_ml [item][Hkv][RPT][2], part_o [item][Hkv][RPT][D], RPT =
// 32 * (query tiles of a unit); counters [sequence][Hkv][q_blocks], zero between launches; queue [8]: next
// position of every XCD's queue, zeroed by the plan kernel for every layer of the step.
// The read-only index arrays arrive as separate __restrict__ arguments (not inside the by-value Plan / KvView
// structs): only then can the compiler prove that the kernel's own stores never alias them, and only then do the
// per-tile block-table lookups stay scalar loads inside the persistent loop.  A vector load of a page id in the
// tile loop must be waited for with vmcnt(0), which serialises the K/V prefetch.
template <int NQ, int QG, int D>
__global__ void __launch_bounds__(256) attn_mfma_kernel(const int32_t* __restrict__ seq_k, const int32_t* __restrict__ seq_c,
                                                        const int32_t* __restrict__ row_start, const int32_t* __restrict__ seq_slot,
                                                        const int32_t* __restrict__ attn_meta, const int32_t* __restrict__ item_start,
                                                        const int32_t* __restrict__ item_seq, const int32_t* __restrict__ item_chunk,
                                                        const int32_t* __restrict__ block_table, int max_pages, int n_pages,
                                                        int n_units, int Hq, int Hkv, float scale_log2e,
                                                        const f16* __restrict__ q, const f16* __restrict__ k_pages,
                                                        const f16* __restrict__ v_pages, f16* __restrict__ out,
                                                        float* __restrict__ part_o, float* __restrict__ part_ml,
                                                        int32_t* __restrict__ counters, int32_t* __restrict__ queue,
                                                        int q_blocks, int32_t* __restrict__ status) {
  constexpr int KS = D / 16;            // MFMA K-steps of the QK^T product
  constexpr int DT = D / 32;            // 32-wide d tiles of the output
  constexpr int RP = 32 * NQ * QG;      // padded query rows per workgroup
  constexpr int WPG = 4 / QG;           // waves per group (token split inside the workgroup)
  constexpr int ROWS_W = 32 * NQ;       // query rows held by one wave
  constexpr int LDO = D + 4;            // row stride (floats) of an accumulator in LDS: 4 banks of skew per row
  extern __shared__ __align__(16) char lds_raw[];
  constexpr int kListMax = 64;          // units with partials waiting for the next flush
  __shared__ int s_list[kListMax];
  __shared__ int s_nlist;
  __shared__ int s_w;

  // Persistent workgroups with one work queue per XCD.  Unit u belongs to XCD u % 8 (workgroup ids are dealt
  // round-robin to the XCDs), and that XCD's queue lists (unit, query block) pairs with the query blocks of a
  // unit next to each other, so they are picked up by workgroups of the same XCD at about the same time and the
  // second reader of the unit's K/V hits L2.  A workgroup starts with the pair at its own position and then
  // takes pairs from the queue (one atomic each) until none is left: units differ in cost (chunk tails, number
  // of draft rows), a static assignment left a quarter of the GPU idle on ragged batches.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, wgs_per_xcd = gridDim.x >> 3;
  const int n_live = min(attn_meta[1] * Hkv, n_units);
  const int total_w = (n_live > xcd ? (n_live - xcd + 7) / 8 : 0) * q_blocks;   // pairs of this XCD
  auto process = [&](const int unit, const int qb) {
  const int item = unit / Hkv, h = unit % Hkv;
  const int b = item_seq[item], chunk = item_chunk[item];
  const int n_ch = item_start[b + 1] - item_start[b];   // chunks of this sequence
  const int qt0 = qb * NQ * QG;                         // first query tile of this workgroup
  const int k = seq_k[b];
  if (k < 0) return;
  const int G = Hq / Hkv;
  const int c = seq_c[b];
  const int n_tok = c + k + 1;
  const int R = (k + 1) * G;
  if (qt0 * 32 >= R) return;                            // this sequence has fewer query rows
  // the wave index is made scalar so that everything derived from it (tile index, block-table lookups)
  // stays on the scalar unit: a vector load of a page id inside the loop would force vmcnt(0) and
  // serialise the K/V prefetch
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int grp = wave / WPG, wig = wave % WPG;
  const int ln = lane & 31, lg = lane >> 5;
  const int row0 = row_start[b];
  const int32_t* __restrict__ bt = block_table + (size_t)seq_slot[b] * max_pages;
  const size_t page_elems = kv_page_elems(Hkv, D);

  // Query fragments (B operand: lane (n, g) holds Q[row n][g*D/2 + 8s + j]) are staged once in LDS in
  // fragment order and re-read per use: keeping them in registers would push the kernel into spills,
  // and a spill reload inside the loop forces vmcnt(0), i.e. it serialises the K/V prefetch.
  u32x4* s_q = (u32x4*)lds_raw;                         // [RP/32][KS][64] (the region is reused by the merge)
  int lim[NQ];                                          // last visible cache position of the lane's row
#pragma unroll
  for (int qt = 0; qt < NQ; ++qt) {
    const int qr = (qt0 + grp * NQ + qt) * 32 + ln;
    lim[qt] = (qr < R) ? c + qr / G : -1;
  }
  const int n_tiles = (n_tok + kTile - 1) / kTile;
  const int cht = attn_meta[0];
  const int t_begin = min(chunk * cht, n_tiles), t_end = min(t_begin + cht, n_tiles);
  const bool group_active = ((qt0 + grp * NQ) * 32) < R;        // wave-uniform
  // tiles of this wave: t0, t0 + WPG, ... (n_my of them)
  const int t0 = t_begin + wig;
  const int n_my = (group_active && t0 < t_end) ? (t_end - t0 + WPG - 1) / WPG : 0;
  const int t_last = t0 + (n_my - 1) * WPG;
  auto tile_offset = [&](int t) -> size_t {
    const int tb = t * kTile;
    const int page = min(max(bt[tb / kPage], 0), n_pages - 1);
    return (size_t)page * page_elems + (size_t)(h * 2 + ((tb / kTile) & 1)) * (kTile * D) + lane * 8;
  };
  auto load_k = [&](size_t off, u32x4 (&kf)[KS]) {
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[s] = *(const u32x4*)(k_pages + off + s * 512);
  };
  auto load_v = [&](size_t off, u32x4 (&vf)[DT * 2]) {
#pragma unroll
    for (int x = 0; x < DT * 2; ++x) vf[x] = *(const u32x4*)(v_pages + off + x * 512);
  };

  // Prologue order: the query fragments are requested first and the first two K/V tiles right behind
  // them, so that staging the queries in LDS only waits for the (older) query loads while 32 KiB of
  // K/V per wave are already in flight.
  constexpr int QF = (RP / 32) * KS / 4;                // query fragments (1 KiB) staged by each wave
  u32x4 qv[QF];
#pragma unroll
  for (int j = 0; j < QF; ++j) {
    const int f = wave + 4 * j;
    const int qtile = f / KS, s = f % KS;
    const int qr = min((qt0 + qtile) * 32 + ln, R - 1);         // clamped rows are never used: their scores are masked
    const int iq = qr / G, hg = qr % G;
    qv[j] = *(const u32x4*)(q + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D + lg * (D / 2) + s * 8);
  }
  // Two K/V tiles live in registers (k0/v0, k1/v1).  A buffer is refilled with the tile two steps
  // ahead as soon as its MFMAs have been issued: K right after the score product, V right after the
  // output product, so between 16 and 32 KiB per wave are in flight at any time and no register
  // copies are needed.  All refills are unconditional (clamped to the wave's last tile).
  u32x4 k0[KS], v0[DT * 2], k1[KS], v1[DT * 2];
  {
    // unconditional (a wave without tiles reads the sequence's last tile and ignores it): loads issued under
    // a branch would make the wait for the query loads above a wait for everything
    const int ta = min(t0, n_tiles - 1), tb = n_my > 1 ? t0 + WPG : ta;
    const size_t oa = tile_offset(ta), ob = tile_offset(tb);
    load_k(oa, k0);
    load_v(oa, v0);
    load_k(ob, k1);
    load_v(ob, v1);
  }
#pragma unroll
  for (int j = 0; j < QF; ++j) s_q[(wave + 4 * j) * 64 + lane] = qv[j];
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

  // One tile: scores from kc, refill kc with tile t_pref, softmax, output product from vc, refill vc.
  auto tile = [&](auto pref, int t, int t_pref, u32x4 (&kc)[KS], u32x4 (&vc)[DT * 2]) {
    constexpr bool PREF = decltype(pref)::value;
    // the block-table entry of the refill tile is requested (scalar load) before the score product, so
    // that its latency is over by the time the refill is issued
    const size_t off_pref = PREF ? tile_offset(t_pref) : 0;
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
    if (PREF) load_k(off_pref, kc);
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
    __builtin_amdgcn_sched_barrier(0);
    if (PREF) load_v(off_pref, vc);
    __builtin_amdgcn_sched_barrier(0);
  };

  {
    int i = 0;
    for (; i + 2 <= n_my; i += 2) {
      const int t = t0 + i * WPG;
      tile(std::true_type{}, t, min(t + 2 * WPG, t_last), k0, v0);
      tile(std::true_type{}, t + WPG, min(t + 3 * WPG, t_last), k1, v1);
    }
    if (i < n_my) tile(std::false_type{}, t0 + i * WPG, 0, k0, v0);
  }
  __syncthreads();                                      // all waves are done with the query fragments

  // ---- merge the waves of each group -----------------------------------------------------------
  // Every wave stores its unscaled accumulator (rows x D, row-major, padded rows) and its per-row
  // (max, sum) in LDS; after ONE barrier all 256 threads combine them: TPR threads per query row, each
  // sums its 16-byte chunks over the waves of the row's group with the usual exp2(m_w - m) weights and
  // writes the result (single chunk: normalised float16 rows; several chunks: float32 partial + (m, l)).
  float* s_o = (float*)lds_raw;                         // [4 waves][ROWS_W][LDO]
  float* s_m = s_o + 4 * ROWS_W * LDO;                  // [4][ROWS_W] per-wave running max
  float* s_l = s_m + 4 * ROWS_W;                        // [4][ROWS_W] per-wave sum
  {
    float* mine = s_o + (size_t)wave * ROWS_W * LDO;
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
      l_run[qt] += __shfl_xor(l_run[qt], 32);
      if (lg == 0) {
        s_m[wave * ROWS_W + qt * 32 + ln] = m_run[qt];
        s_l[wave * ROWS_W + qt * 32 + ln] = l_run[qt];
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *(f32x4*)(mine + (qt * 32 + ln) * LDO + dt * 32 + 8 * i4 + 4 * lg) =
              f32x4{o[qt][dt][4 * i4], o[qt][dt][4 * i4 + 1], o[qt][dt][4 * i4 + 2], o[qt][dt][4 * i4 + 3]};
    }
  }
  __syncthreads();
  {
    constexpr int TPR = 256 / RP;                       // threads per query row
    constexpr int CH = D / 4;                           // 16-byte chunks per row
    const int wr = threadIdx.x / TPR, sub = threadIdx.x % TPR;
    const int g = wr / ROWS_W, lr = wr % ROWS_W;
    const int qr = qt0 * 32 + wr;
    if (qr < R) {
      float mw[WPG], mt = -INFINITY;
#pragma unroll
      for (int w = 0; w < WPG; ++w) {
        mw[w] = s_m[(g * WPG + w) * ROWS_W + lr];
        mt = fmaxf(mt, mw[w]);
      }
      const float ms = (mt == -INFINITY) ? 0.f : mt;
      float lt = 0.f;
#pragma unroll
      for (int w = 0; w < WPG; ++w) {
        mw[w] = __builtin_amdgcn_exp2f(mw[w] - ms);      // weight of wave w (0 for a wave that saw no token)
        lt += s_l[(g * WPG + w) * ROWS_W + lr] * mw[w];
      }
      const int iq = qr / G, hg = qr % G;
      const float inv = 1.0f / lt;                      // row i always sees at least position c + i: lt > 0
      f16* dst = out + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D;
      const size_t pr = ((size_t)(item_start[b] + chunk) * Hkv + h) * ((size_t)RP * q_blocks) + qr;   // slot of (sequence, chunk, head)
#pragma unroll
      for (int j = 0; j < CH / TPR; ++j) {
        const int ch = sub + j * TPR;
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < WPG; ++w) {
          const f32x4 v = *(const f32x4*)(s_o + ((size_t)(g * WPG + w) * ROWS_W + lr) * LDO + ch * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[e] += v[e] * mw[w];
        }
        if (n_ch == 1) {
          *(f16x4*)(dst + ch * 4) = to_f16x4_guarded(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv, status);
        } else {
          *(f32x4*)(part_o + pr * D + ch * 4) = acc;
        }
      }
      if (n_ch > 1 && sub == 0) { part_ml[pr * 2] = mt; part_ml[pr * 2 + 1] = lt; }
    }
    // several chunks: remember the unit; its partial is published and merged in flush() below
    if (n_ch > 1 && threadIdx.x == 0) { s_list[s_nlist] = unit * q_blocks + qb; s_nlist = s_nlist + 1; }
  }
  };   // process

  // Merge of the units with several chunks: the LAST workgroup of (sequence, KV head, query block) to publish
  // its partial merges all of them; nobody waits.  Release: the workgroup's partial stores are made visible
  // device-wide (one fence for all units in the list: a fence per unit, i.e. an L2 write-back and invalidate
  // each, cost more than the attention itself on ragged batches) before the counters are bumped; acquire: a
  // workgroup that reads n_ch - 1 sees the partials of all the others.
  auto merge_unit = [&](const int unit, const int qb) {
    const int item = unit / Hkv, h = unit % Hkv;
    const int b = item_seq[item];
    const int n_ch = item_start[b + 1] - item_start[b];
    const int G = Hq / Hkv, R = (seq_k[b] + 1) * G, row0 = row_start[b];
    constexpr int TPR = 256 / RP, CH = D / 4;
    const int wr = threadIdx.x / TPR, sub = threadIdx.x % TPR;
    const int qr = qb * RP + wr;
    if (qr >= R) return;
    const size_t rpt = (size_t)RP * q_blocks;
    const size_t u0 = (size_t)item_start[b] * Hkv + h;           // unit of chunk 0; chunk c is Hkv units further
    float mt = -INFINITY;
    for (int c = 0; c < n_ch; ++c) mt = fmaxf(mt, part_ml[((u0 + (size_t)c * Hkv) * rpt + qr) * 2]);
    float lt = 0.f;
    f32x4 acc[CH / TPR];
#pragma unroll
    for (int j = 0; j < CH / TPR; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < n_ch; ++c) {
      const size_t pc = (u0 + (size_t)c * Hkv) * rpt + qr;
      const float m = part_ml[pc * 2];
      if (m == -INFINITY) continue;
      const float f = __builtin_amdgcn_exp2f(m - mt);
      lt += part_ml[pc * 2 + 1] * f;
#pragma unroll
      for (int j = 0; j < CH / TPR; ++j) {
        const f32x4 v = *(const f32x4*)(part_o + pc * D + (sub + j * TPR) * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[j][e] += v[e] * f;
      }
    }
    const int iq = qr / G, hg = qr % G;
    const float inv = 1.0f / lt;
    f16* dst = out + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D;
#pragma unroll
    for (int j = 0; j < CH / TPR; ++j)
      *(f16x4*)(dst + (sub + j * TPR) * 4) =
          to_f16x4_guarded(acc[j][0] * inv, acc[j][1] * inv, acc[j][2] * inv, acc[j][3] * inv, status);
  };
  auto flush = [&]() {
    __syncthreads();
    const int n = s_nlist;
    if (n == 0) return;                                 // uniform
    __threadfence();
    __syncthreads();
    if ((int)threadIdx.x < n) {
      const int unit = s_list[threadIdx.x] / q_blocks, qb = s_list[threadIdx.x] % q_blocks;
      const int item = unit / Hkv, h = unit % Hkv, b = item_seq[item];
      const int n_ch = item_start[b + 1] - item_start[b];
      int32_t* cnt = counters + ((size_t)b * Hkv + h) * q_blocks + qb;
      const int old = atomicAdd(cnt, 1);
      const bool last = old == n_ch - 1;
      if (last) *cnt = 0;                               // ready for the next launch (stream order)
      else s_list[threadIdx.x] = -1;
    }
    __syncthreads();
    __threadfence();
    for (int i = 0; i < n; ++i)
      if (s_list[i] >= 0) merge_unit(s_list[i] / q_blocks, s_list[i] % q_blocks);
    __syncthreads();
    if (threadIdx.x == 0) s_nlist = 0;
  };

  if (threadIdx.x == 0) s_nlist = 0;
  int w = slot;                                         // position in this XCD's queue
  while (w < total_w) {
    __syncthreads();                                    // LDS of the previous unit is no longer read
    if (s_nlist == kListMax) flush();
    process(xcd + 8 * (w / q_blocks), w % q_blocks);
    if (total_w <= wgs_per_xcd) break;                  // at most one pair per workgroup: nothing to take
    __syncthreads();
    if (threadIdx.x == 0) s_w = atomicAdd(queue + xcd, 1) + wgs_per_xcd;
    __syncthreads();
    w = __builtin_amdgcn_readfirstlane(s_w);         // keeps everything derived from it on the scalar unit
  }
  flush();
}

static int rows_padded(const Shape& s, int k_max) {
  int R = (k_max + 1) * (s.Hq / s.Hkv);
  int tiles = (R + 31) / 32;
  if (tiles <= 2) return tiles * 32;
  return 128;
}

// Scratch: completion counters [B_max][Hkv][4], then (max, sum) and float32 partial rows of every unit
// (work item x KV head) at the largest work-list capacity.
static size_t counters_bytes(const Shape& s, int B_max) { return ((size_t)B_max * s.Hkv * 4 * sizeof(int32_t) + 255) / 256 * 256; }

size_t attention_scratch_bytes(const Shape& s, int B_max, int k_max) {
  if (s.dtype != BS_BF16) return 256;
  const size_t rp = rows_padded(s, k_max);
  const size_t units = (size_t)attn_item_capacity(B_max, kAttnMaxSmin) * s.Hkv;
  return counters_bytes(s, B_max) + units * rp * (s.D + 2) * sizeof(float);
}

// Test hook, not part of the public ABI: forces the launch shape of the bf16 attention kernel (0 = choose
// automatically) so that every instantiation can be exercised at small batch sizes: q_blocks = query blocks
// per (sequence, KV head) (ignored if it does not divide the number of query tiles), n_chunks = token chunks
// of the longest sequence.
static int g_force_q_blocks = 0, g_force_n_chunks = 0;
extern "C" void bs_debug_attention_shape(int q_blocks, int n_chunks) {
  g_force_q_blocks = q_blocks;
  g_force_n_chunks = n_chunks;
}

// Shape of the launch.  A unit = (sequence, KV head) has `tiles` query tiles of 32 rows.  With enough units to
// fill the 256 CUs one workgroup takes all tiles of a unit (K/V fragments are loaded once and used for every
// tile); with fewer units the query tiles are spread over q_blocks workgroups (the extra readers hit L2).  What
// is still missing to reach ~256 workgroups, and the balance between sequences of different length, comes from
// the token chunks of the work list, which the plan kernel sizes on the device from s_min = wanted (sequence,
// chunk) items.
static void launch_shape(const Shape& s, int B, int k_max, int& q_blocks, int& s_min, int& force_chunks) {
  const int tiles = rows_padded(s, k_max) / 32;                    // 1, 2 or 4
  const int units = B * s.Hkv;
  q_blocks = 1;
  if (tiles == 2 && units < 256) q_blocks = 2;
  // four tiles: one workgroup of eight waves per unit (attn_wide_kernel), every wave one query tile, K/V shared
  // through LDS.  (Before: two query blocks of two tiles each, four waves, the second reader served by L2; measured
  // on the ragged batch of 128 sequences, 7B heads: 620 us per layer, matrix unit busy 10 %, waves waiting 36 %.)
  const int qb_forced = g_force_q_blocks;
  if (qb_forced >= 1 && qb_forced <= tiles && tiles % qb_forced == 0) q_blocks = qb_forced;
  s_min = (256 + s.Hkv * q_blocks - 1) / (s.Hkv * q_blocks);
  if (s_min > kAttnMaxSmin) s_min = kAttnMaxSmin;
  force_chunks = g_force_n_chunks;
}

void attention_plan_params(const Shape& s, int B, int k_max, int* s_min, int* force_chunks) {
  if (s.dtype != BS_BF16) { *s_min = 0; *force_chunks = 0; return; }
  int q_blocks;
  launch_shape(s, B, k_max, q_blocks, *s_min, *force_chunks);
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}
void launch_attention_init(const Shape& s, int B_max, void* scratch, hipStream_t st) {
  if (s.dtype != BS_BF16) return;
  const int n = (int)(counters_bytes(s, B_max) / sizeof(int32_t));
  hipLaunchKernelGGL(zero_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, (int32_t*)scratch, n);
}

template <int NQ, int QG, int D>
static void launch_mfma_attn(const Shape& s, const Plan& p, const KvView& kv, int layer, int B, int B_max, int M_max, const void* q,
                             const void* k_pages, const void* v_pages, void* out, void* scratch, int q_blocks,
                             int s_min, void* prof_token, hipStream_t st) {
  constexpr int RP = 32 * NQ * QG;
  const int rpt = RP * q_blocks;                                       // padded query rows of a unit
  size_t lds = (size_t)4 * 32 * NQ * (D + 4) * 4 + 2 * 4 * 32 * NQ * 4;   // accumulators of 4 waves + statistics
  const size_t lds_q = (size_t)(RP / 32) * (D / 16) * 1024;           // query fragments (same region, earlier)
  if (lds < lds_q) lds = lds_q;
  const int n_units = attn_item_capacity(B, s_min) * s.Hkv;
  int32_t* counters = (int32_t*)scratch;
  float* part_ml = (float*)((char*)scratch + counters_bytes(s, B_max));
  float* part_o = part_ml + (size_t)n_units * rpt * 2;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  auto kern = attn_mfma_kernel<NQ, QG, D>;
  static bool attr_set = false;
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr_set = true; }
  // one workgroup per CU (every instantiation for head size 128 needs more than half of a CU's registers);
  // fewer when the work list cannot be longer
  const int cap_w = (n_units * q_blocks + 7) / 8 * 8;
  const int grid = cap_w < 256 ? cap_w : 256;
  if (prof_token) attention_prof_mark(prof_token, st, true);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, st, p.seq_k, p.seq_c, p.row_start, p.seq_slot, p.attn_meta,
                     p.item_start, p.item_seq, p.item_chunk, kv.block_table, kv.max_pages, kv.n_pages, n_units, s.Hq,
                     s.Hkv, scale_log2e, (const f16*)q,
                     (const f16*)k_pages, (const f16*)v_pages, (f16*)out, part_o, part_ml, counters, p.attn_queue + 8 * layer, q_blocks,
                     p.status);
  if (prof_token) attention_prof_mark(prof_token, st, false);
}

template <int D>
static void launch_wide_attn(const Shape& s, const Plan& p, const KvView& kv, int layer, int B, int B_max, const void* q,
                             const void* k_pages, const void* v_pages, void* out, void* scratch, int s_min,
                             void* prof_token, hipStream_t st) {
  constexpr int NF = D / 16 + 2 * (D / 32);
  size_t lds = (size_t)8 * 32 * (D + 4) * 4 + 2 * 8 * 32 * 4;          // merge: accumulators of 8 waves + statistics
  const size_t lds_kv = (size_t)2 * 4 * NF * 1024;                     // two buffers x four phases (two query tiles)
  if (lds < lds_kv) lds = lds_kv;
  const int n_units = attn_item_capacity(B, s_min) * s.Hkv;
  float* part_ml = (float*)((char*)scratch + counters_bytes(s, B_max));
  float* part_o = part_ml + (size_t)n_units * 128 * 2;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)D);
  auto kern = attn_wide_kernel<D>;
  static bool attr_set = false;
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr_set = true; }
  const int cap_w = (n_units + 7) / 8 * 8;
  const int grid = cap_w < 256 ? cap_w : 256;                          // one workgroup of eight waves per CU
  if (prof_token) attention_prof_mark(prof_token, st, true);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(512), lds, st, p.seq_k, p.seq_c, p.row_start, p.seq_slot, p.attn_meta,
                     p.item_start, p.item_seq, p.item_chunk, kv.block_table, kv.max_pages, kv.n_pages, n_units, s.Hq,
                     s.Hkv, scale_log2e, (const f16*)q, (const f16*)k_pages, (const f16*)v_pages, (f16*)out, part_o,
                     part_ml, p.attn_queue + 8 * layer, p.status);
  hipLaunchKernelGGL(attn_wide_merge_kernel<D>, dim3(B * s.Hkv), dim3(512), 0, st, p.seq_k, p.row_start, p.item_start, s.Hq,
                     s.Hkv, part_o, part_ml, (f16*)out, p.status);
  if (prof_token) attention_prof_mark(prof_token, st, false);
}

void launch_attention(const Shape& s, const Plan& p, const KvView& kv, int layer, int B, int B_max, int k_max, int M_max,
                      const void* q, const void* k_pages, const void* v_pages, void* out, void* scratch,
                      void* prof_token, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)s.D);
  if (s.dtype == BS_F32) {
    hipLaunchKernelGGL((attn_simple_kernel<float, float>), dim3(M_max, s.Hq), dim3(256), 0, st, p, kv, s.Hq, s.Hkv, s.D, scale,
                       (const float*)q, (const float*)k_pages, (const float*)v_pages, (float*)out);
    return;
  }
  int q_blocks, s_min, force_chunks;
  launch_shape(s, B, k_max, q_blocks, s_min, force_chunks);
  const int tiles_wg = rows_padded(s, k_max) / 32 / q_blocks;      // query tiles per workgroup: 1, 2 or 4
#define BS_ATTN(NQ, QG)                                                                                         \
  do {                                                                                                          \
    if (s.D == 128) launch_mfma_attn<NQ, QG, 128>(s, p, kv, layer, B, B_max, M_max, q, k_pages, v_pages, out, scratch, q_blocks, s_min, prof_token, st); \
    else launch_mfma_attn<NQ, QG, 64>(s, p, kv, layer, B, B_max, M_max, q, k_pages, v_pages, out, scratch, q_blocks, s_min, prof_token, st);   \
  } while (0)
  if (tiles_wg == 1) BS_ATTN(1, 1);
  else if (tiles_wg == 2) BS_ATTN(2, 1);
  else if (s.D == 128) launch_wide_attn<128>(s, p, kv, layer, B, B_max, q, k_pages, v_pages, out, scratch, s_min, prof_token, st);
  else launch_wide_attn<64>(s, p, kv, layer, B, B_max, q, k_pages, v_pages, out, scratch, s_min, prof_token, st);
#undef BS_ATTN
}
