// Verify attention for batches in which a sequence may have three or four 32-row query tiles per KV head
// ((k_b + 1) * G > 64 query rows: long draft blocks on wide GQA groups, Sec. 3.3's "unified" launch at its
// widest).  Same work list, page layout, partial results and last-arriver merge as attn_mfma_kernel in
// attention.hip; what differs is how a workgroup spends a CU.
//
// With four query tiles the step is no longer a pure stream: per 32-token K/V tile (16 KiB at head size 128) a
// CU owes 64 MFMAs and four softmax passes.  One wave per SIMD that owns two query tiles (the narrow kernel) issues
// ~21 vector instructions per MFMA and then waits for its own loads: measured on the long-tail batch, the matrix
// unit was busy 10 % of the time, the waves waited 36 % of it, and the kernel reached 2.5 TB/s although L2 served
// the second reader of every tile (fetched bytes 1.07 x algorithmic).  Here a workgroup has EIGHT waves, two per
// SIMD, so that one wave's softmax and LDS traffic overlap the other's MFMAs and waits, and every wave owns ONE
// query tile (64 accumulator registers), which is what lets two waves share a SIMD's 512 registers:
//   * wave w = (query tile qt = w % NQT, token phase ph = w / NQT), NQT = 2 or 4 query tiles per unit; the 8 / NQT
//     phases work on different token tiles of the chunk at the same time;
//   * the NQT waves of a phase share one K/V tile through LDS: each loads 1 / NQT of its 1 KiB fragments
//     (HBM -> registers -> LDS, the page layout is already fragment order, so the LDS image is a straight copy and
//     every ds_read_b128 / ds_write_b128 is a conflict-free 1 KiB sweep), so K/V leave HBM once per unit whatever
//     the number of query tiles, with no reliance on L2;
//   * two LDS buffers per phase and one register stage: in iteration i a wave writes its share of tile i + 1 to
//     the other buffer, requests its share of tile i + 2, computes on tile i, then all eight waves meet at one
//     barrier; loads are in flight for more than a full iteration;
//   * query fragments stay in registers (one tile: 32 registers at head size 128).
// Units with one query tile run as NQT = 2 with the second wave of each pair only loading.
#pragma once
#include "gemm_mfma.h"

template <int D>
__global__ void __launch_bounds__(512) attn_wide_kernel(const int32_t* __restrict__ seq_k, const int32_t* __restrict__ seq_c,
                                                        const int32_t* __restrict__ row_start, const int32_t* __restrict__ seq_slot,
                                                        const int32_t* __restrict__ attn_meta, const int32_t* __restrict__ item_start,
                                                        const int32_t* __restrict__ item_seq, const int32_t* __restrict__ item_chunk,
                                                        const int32_t* __restrict__ block_table, int max_pages, int n_pages,
                                                        int n_units, int Hq, int Hkv, float scale_log2e,
                                                        const f16* __restrict__ q, const f16* __restrict__ k_pages,
                                                        const f16* __restrict__ v_pages, f16* __restrict__ out,
                                                        float* __restrict__ part_o, float* __restrict__ part_ml,
                                                        int32_t* __restrict__ queue, int32_t* __restrict__ status) {
  constexpr int KS = D / 16;            // MFMA K-steps of the QK^T product = K fragments of a tile
  constexpr int DT = D / 32;            // 32-wide d tiles of the output; V fragments of a tile = 2 DT
  constexpr int NF = KS + 2 * DT;       // 1 KiB fragments of one K/V tile
  constexpr int RPT = 128;              // padded query rows of a unit (stride of the partial results)
  constexpr int LDO = D + 4;            // row stride (floats) of an accumulator in LDS: 4 banks of skew per row
  constexpr int THREADS = 512;
  extern __shared__ __align__(16) char lds_raw[];
  __shared__ int s_w;

  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, wgs_per_xcd = gridDim.x >> 3;
  const int n_live = min(attn_meta[1] * Hkv, n_units);
  const int total_w = n_live > xcd ? (n_live - xcd + 7) / 8 : 0;   // units of this XCD (unit u belongs to XCD u % 8)
  // the wave index is made scalar so that everything derived from it stays on the scalar unit
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int ln = lane & 31, lg = lane >> 5;
  const size_t page_elems = kv_page_elems(Hkv, D);

  // One unit with NQT query tiles (2 or 4).
  auto run = [&](auto nqt_tag, const int unit) {
    constexpr int NQT = decltype(nqt_tag)::value;
    constexpr int NPH = 8 / NQT;        // token phases
    constexpr int LPW = NF / NQT;       // fragments a wave moves per tile
    const int item = unit / Hkv, h = unit % Hkv;
    const int b = item_seq[item], chunk = item_chunk[item];
    const int n_ch = item_start[b + 1] - item_start[b];
    const int k = seq_k[b];
    const int G = Hq / Hkv;
    const int c = seq_c[b];
    const int n_tok = c + k + 1;
    const int R = (k + 1) * G;
    const int row0 = row_start[b];
    const int32_t* __restrict__ bt = block_table + (size_t)seq_slot[b] * max_pages;
    const int qt = wave % NQT, ph = wave / NQT;
    const bool has_rows = qt * 32 < R;                   // wave-uniform: a wave without query rows only moves data
    const int n_tiles = (n_tok + kTile - 1) / kTile;
    const int cht = attn_meta[0];
    const int t_begin = min(chunk * cht, n_tiles), t_end = min(t_begin + cht, n_tiles);
    const int n_it = (t_end - t_begin + NPH - 1) / NPH;  // iterations of the workgroup (at least 1: chunks are not empty)
    auto tile_of = [&](int i) { return t_begin + ph + NPH * i; };
    auto tile_offset = [&](int t) -> size_t {            // element offset of this lane's 16 bytes in fragment 0 of tile t
      const int tb = min(t, n_tiles - 1) * kTile;        // clamped: a phase without a tile re-reads the last one
      const int page = min(max(bt[tb / kPage], 0), n_pages - 1);
      return (size_t)page * page_elems + (size_t)(h * 2 + ((tb / kTile) & 1)) * (kTile * D) + lane * 8;
    };
    char* const my_stage = lds_raw + (size_t)ph * NF * 1024 + lane * 16;      // buffer 0 of this phase
    constexpr int BUF_BYTES = NPH * NF * 1024;
    u32x4 stg[LPW];
    auto load_share = [&](int t) {
      const size_t off = tile_offset(t);
#pragma unroll
      for (int j = 0; j < LPW; ++j) {
        const int f = qt + NQT * j;
        stg[j] = (f < KS) ? *(const u32x4*)(k_pages + off + f * 512) : *(const u32x4*)(v_pages + off + (f - KS) * 512);
      }
    };
    auto store_share = [&](int buf) {
#pragma unroll
      for (int j = 0; j < LPW; ++j) *(u32x4*)(my_stage + buf * BUF_BYTES + (qt + NQT * j) * 1024) = stg[j];
    };

    // query fragments of this wave's tile (B operand: lane (n, g) holds Q[row n][g*D/2 + 8s + j]); rows beyond R are
    // clamped and masked through lim
    const int qr = qt * 32 + ln;
    const int lim = (qr < R) ? c + qr / G : -1;
    u32x4 qf[KS];
    {
      const int qc = min(qr, R - 1);
      const int iq = qc / G, hg = qc % G;
      const f16* src = q + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D + lg * (D / 2);
#pragma unroll
      for (int s = 0; s < KS; ++s) qf[s] = *(const u32x4*)(src + s * 8);
    }
    load_share(tile_of(0));
    store_share(0);
    load_share(tile_of(1));
    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    __syncthreads();

    for (int i = 0; i < n_it; ++i) {
      store_share((i + 1) & 1);                          // tile i + 1 (requested one iteration ago) -> the other buffer
      if (i + 2 < n_it) load_share(tile_of(i + 2));      // workgroup-uniform
      const int t = tile_of(i);
      if (has_rows && t < t_end) {
        const char* stage = my_stage + (i & 1) * BUF_BYTES;
        const int tok0 = t * kTile + 16 * lg;            // accumulator register r <-> token tok0 + r
        const bool full = (t + 1) * kTile - 1 <= c;      // every token visible to every row: no masking
        // the K fragments are requested from LDS together, before the first product (left to itself the compiler
        // reuses one register quad and waits for every read in turn: eight exposed LDS latencies per product);
        // the V fragments are requested into the same registers once the score products are issued and arrive
        // while the softmax runs
        u32x4 kf[KS], vf[2 * DT];
#pragma unroll
        for (int s = 0; s < KS; ++s) kf[s] = *(const u32x4*)(stage + s * 1024);
        __builtin_amdgcn_sched_barrier(0);
        f32x16 st;
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s)
          st = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(kf[s]), as_f16x8(qf[s]), st, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x2 = 0; x2 < 2 * DT; ++x2) vf[x2] = *(const u32x4*)(stage + (KS + x2) * 1024);
        __builtin_amdgcn_sched_barrier(0);
        float x[16];
        if (full) {
#pragma unroll
          for (int r = 0; r < 16; ++r) x[r] = st[r];
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) x[r] = (tok0 + r <= lim) ? st[r] : -INFINITY;
        }
        float mloc = x[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mloc = fmaxf(mloc, x[r]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32)) * scale_log2e;       // scale > 0 commutes with max
        const float m_new = fmaxf(m_run, mloc);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          x[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[r], scale_log2e, -m_safe));   // exp2(-inf) = 0
          psum += x[r];
        }
        l_run = l_run * alpha + psum;                    // per lane half; halves are added at the end
        m_run = m_new;
        if (__any(alpha != 1.0f)) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        }
        f16x8 pf[2];
#pragma unroll
        for (int j = 0; j < 8; ++j) { pf[0][j] = (f16)x[j]; pf[1][j] = (f16)x[8 + j]; }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(vf[dt * 2 + t2]), pf[t2], o[dt], 0, 0, 0);
      }
      __syncthreads();                                   // buffer i & 1 is free, buffer (i + 1) & 1 is complete
    }

    // ---- merge the NPH phases of each query tile through LDS (the K/V buffers are free after the loop's last
    // barrier): every wave stores its unscaled accumulator and its per-row (max, sum); after one barrier the 512
    // threads combine them, TPR threads per query row.
    float* s_o = (float*)lds_raw;                        // [8 waves][32][LDO]
    float* s_m = s_o + 8 * 32 * LDO;                     // [8][32]
    float* s_l = s_m + 8 * 32;
    {
      float* mine = s_o + (size_t)wave * 32 * LDO;
      l_run += __shfl_xor(l_run, 32);
      if (lg == 0) { s_m[wave * 32 + ln] = m_run; s_l[wave * 32 + ln] = l_run; }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *(f32x4*)(mine + ln * LDO + dt * 32 + 8 * i4 + 4 * lg) =
              f32x4{o[dt][4 * i4], o[dt][4 * i4 + 1], o[dt][4 * i4 + 2], o[dt][4 * i4 + 3]};
    }
    __syncthreads();
    {
      constexpr int TPR = THREADS / (32 * NQT);          // threads per query row: 8 or 4
      constexpr int CH = D / 4;                          // 16-byte chunks per row
      const int wr = threadIdx.x / TPR, sub = threadIdx.x % TPR;      // wr = query row of the unit, 0 .. 32 NQT - 1
      const int tq = wr / 32, lr = wr % 32;
      if (wr < R) {
        float mw[NPH], mt = -INFINITY;
#pragma unroll
        for (int w = 0; w < NPH; ++w) {
          mw[w] = s_m[(w * NQT + tq) * 32 + lr];
          mt = fmaxf(mt, mw[w]);
        }
        const float ms = (mt == -INFINITY) ? 0.f : mt;
        float lt = 0.f;
#pragma unroll
        for (int w = 0; w < NPH; ++w) {
          mw[w] = __builtin_amdgcn_exp2f(mw[w] - ms);    // weight of phase w (0 for a phase that saw no token)
          lt += s_l[(w * NQT + tq) * 32 + lr] * mw[w];
        }
        const int iq = wr / G, hg = wr % G;
        const float inv = 1.0f / lt;                     // a single-chunk row always sees position c + i: lt > 0
        f16* dst = out + (size_t)(row0 + iq) * Hq * D + (size_t)(h * G + hg) * D;
        const size_t pr = ((size_t)(item_start[b] + chunk) * Hkv + h) * RPT + wr;   // slot of (sequence, chunk, head)
#pragma unroll
        for (int j = 0; j < CH / TPR; ++j) {
          const int ch = sub + j * TPR;
          f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int w = 0; w < NPH; ++w) {
            const f32x4 v = *(const f32x4*)(s_o + ((size_t)(w * NQT + tq) * 32 + lr) * LDO + ch * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += v[e] * mw[w];
          }
          if (n_ch == 1) *(f16x4*)(dst + ch * 4) = to_f16x4_guarded(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv, status);
          else *(f32x4*)(part_o + pr * D + ch * 4) = acc;
        }
        if (n_ch > 1 && sub == 0) { part_ml[pr * 2] = mt; part_ml[pr * 2 + 1] = lt; }
      }
    }
  };   // run

  auto process = [&](const int unit) {
    const int b = item_seq[unit / Hkv];
    const int k = seq_k[b];
    if (k < 0) return;                                   // workgroup-uniform
    if ((k + 1) * (Hq / Hkv) > 64) run(std::integral_constant<int, 4>{}, unit);
    else run(std::integral_constant<int, 2>{}, unit);
  };

  int w = slot;                                         // position in this XCD's queue
  while (w < total_w) {
    __syncthreads();                                    // LDS of the previous unit is no longer read
    process(xcd + 8 * w);
    if (total_w <= wgs_per_xcd) break;                  // at most one unit per workgroup: nothing to take
    __syncthreads();
    if (threadIdx.x == 0) s_w = atomicAdd(queue + xcd, 1) + wgs_per_xcd;
    __syncthreads();
    w = __builtin_amdgcn_readfirstlane(s_w);
  }
}

// Second, small launch of the wide path: one workgroup per (sequence, KV head) combines the partial results of a
// sequence that was cut into several chunks (float32 rows + (max, sum) per chunk, slot-addressed) into the final
// float16 rows; sequences with one chunk were written by attn_wide_kernel itself and their workgroups exit at once.
// (Merging inside the attention kernel by the last workgroup to arrive, as attn_mfma_kernel does, needs a
// device-scope fence per publication: once per unit it tripled the kernel's time on the long-tail batch, once per
// workgroup it left every merge to the end of the kernel, 80 us mean / 118 us worst per workgroup with nothing
// streaming meanwhile.  The kernel boundary orders the partial results for free.)
template <int D>
__global__ void __launch_bounds__(512) attn_wide_merge_kernel(const int32_t* __restrict__ seq_k, const int32_t* __restrict__ row_start,
                                                              const int32_t* __restrict__ item_start, int Hq, int Hkv,
                                                              const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                              f16* __restrict__ out, int32_t* __restrict__ status) {
  constexpr int RPT = 128, TPR = 512 / RPT, CH = D / 4, CPT = CH / TPR;   // 4 threads per row, CPT 16-byte chunks each
  const int b = blockIdx.x / Hkv, h = blockIdx.x % Hkv;
  const int n_ch = item_start[b + 1] - item_start[b];
  const int k = seq_k[b];
  if (n_ch <= 1 || k < 0) return;
  const int G = Hq / Hkv, R = (k + 1) * G;
  const int qr = threadIdx.x / TPR, sub = threadIdx.x % TPR;
  if (qr >= R) return;
  const size_t u0 = (size_t)item_start[b] * Hkv + h;             // slot of chunk 0; chunk c is Hkv slots further
  float mt = -INFINITY;
  for (int cc = 0; cc < n_ch; ++cc) mt = fmaxf(mt, part_ml[((u0 + (size_t)cc * Hkv) * RPT + qr) * 2]);
  float lt = 0.f;
  f32x4 acc[CPT];
#pragma unroll
  for (int j = 0; j < CPT; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  // two chunks per round: their loads are requested together (chunk order of the sums is kept)
  for (int c0 = 0; c0 < n_ch; c0 += 2) {
    float m2[2], l2[2];
    f32x4 v[2][CPT];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const size_t pc = (u0 + (size_t)min(c0 + u, n_ch - 1) * Hkv) * RPT + qr;
      m2[u] = part_ml[pc * 2];
      l2[u] = part_ml[pc * 2 + 1];
#pragma unroll
      for (int j = 0; j < CPT; ++j) v[u][j] = *(const f32x4*)(part_o + pc * D + (sub + j * TPR) * 4);
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (c0 + u >= n_ch || m2[u] == -INFINITY) continue;
      const float f = __builtin_amdgcn_exp2f(m2[u] - mt);
      lt += l2[u] * f;
#pragma unroll
      for (int j = 0; j < CPT; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[j][e] += v[u][j][e] * f;
    }
  }
  const int iq = qr / G, hg = qr % G;
  const float inv = 1.0f / lt;
  f16* dst = out + (size_t)(row_start[b] + iq) * Hq * D + (size_t)(h * G + hg) * D;
#pragma unroll
  for (int j = 0; j < CPT; ++j)
    *(f16x4*)(dst + (sub + j * TPR) * 4) =
        to_f16x4_guarded(acc[j][0] * inv, acc[j][1] * inv, acc[j][2] * inv, acc[j][3] * inv, status);
}
