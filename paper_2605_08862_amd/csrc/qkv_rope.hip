// QKV projection fused with the rotary embedding and the tentative KV append (bf16 models, head size 128).
//
//   [M, d] x [ (Hq + 2 Hkv) * 128, d ]^T, then per head: q and k rotated at the row's absolute position
//   (pairs (j, j + 64)), q stored as float16 rows (attention operand), k and v rounded to bf16 and written
//   into the slot's KV page in the page layout.
//
// One workgroup = 32*MT rows x one head: its four waves hold 32 columns each, so the 128 columns of the
// tile are exactly the head and the partner of column j (< 64) sits in the wave two places further.  After
// the main loop (full K, no split) the waves exchange their accumulators through LDS once, rotate with the
// step's cos / sin table and store the final values: the float32 projection never goes to memory and q, k,
// v are still rounded exactly once, after the rotation.  Replaces a split-K GEMM + a separate rotary kernel
// that had to sum the float32 slabs (13.5 + 8 us at M = 576, d = 1536 against about 15 us fused).
#include "gemm_mfma.h"

namespace {
constexpr int kD = 128;

template <int MT>
__global__ void __launch_bounds__(256, (MT <= 2 ? 2 : 1))
qkv_rope_kernel(Plan p, KvView kv, int M_max, int K, int Hq, int Hkv, const f16* __restrict__ A,
                const f16* __restrict__ Wp, const float* __restrict__ cos_t, const float* __restrict__ sin_t,
                f16* __restrict__ q_out, f16* __restrict__ k_pages, f16* __restrict__ v_pages, int m_blocks,
                int defer_rows) {
  using G = MfmaGemm<MT, 1, true>;
  extern __shared__ __align__(16) char lds[];
  // a one-round launch does not wait for the row count before its first loads: it multiplies all M_max rows (those
  // beyond the count are stale rows, each affecting only its own output) and applies the count to the stores
  int M = defer_rows ? M_max : min(p.n_rows[0], M_max);
  // Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2): every XCD takes a contiguous range
  // of (head, M block) tiles, M block fastest, so a head's weights are fetched by one L2 only.
  const int total = m_blocks * (Hq + 2 * Hkv), per_xcd = (total + 7) / 8;
  const int tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (blockIdx.x / 8 >= per_xcd || tile >= total) return;
  const int mb = tile % m_blocks, head = tile / m_blocks;
  const int m0 = mb * G::BM;
  if (m0 >= M) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ln = lane & 31, lg = lane >> 5;
  const int nk = K / kBK;

  typename G::Operands op;
#pragma unroll
  for (int i = 0; i < MT; ++i) {
    int row, g, s;
    G::chunk_of(i, row, g, s);
    const int r = min(m0 + row, M - 1);
    op.x_rows[i] = A + (size_t)r * K + g * 32 + s * 8;
    op.x_lds[i] = G::chunk_lds_offset(row, g, s);
  }
  op.w_tiles[0] = Wp + (size_t)(head * 4 + wave) * nk * kWBlock + lane * 8;
  f32x16 acc[MT][1];
#pragma unroll
  for (int mi = 0; mi < MT; ++mi)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mi][0][i] = 0.f;
  G::run(acc, op, 0, nk, lds);
  if (defer_rows) M = min(p.n_rows[0], M_max);

  // ---- epilogue.  Accumulator register i of lane (ln, lg) in tile mi: row m0 + 32 mi + ln,
  // head column d = 32 wave + 8 (i / 4) + 4 lg + (i % 4).
  const bool is_v = head >= Hq + Hkv;
  constexpr int LDX = kD + 4;                         // padded row (floats) of the exchange buffer
  float* s_x = (float*)lds;                           // [32 MT][LDX]; the loop's last barrier has been passed
  if (!is_v) {
    __syncthreads();                                  // every wave is done reading the loop's LDS stages
#pragma unroll
    for (int mi = 0; mi < MT; ++mi)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
        *(f32x4*)(s_x + (mi * 32 + ln) * LDX + 32 * wave + 8 * i4 + 4 * lg) =
            f32x4{acc[mi][0][4 * i4], acc[mi][0][4 * i4 + 1], acc[mi][0][4 * i4 + 2], acc[mi][0][4 * i4 + 3]};
    __syncthreads();
  }
  const float sign = (wave < 2) ? -1.0f : 1.0f;       // y1 = x1 c - x2 s (columns < 64), y2 = x2 c + x1 s
  const int partner = (wave < 2) ? 64 : -64;
#pragma unroll
  for (int mi = 0; mi < MT; ++mi) {
    const int m = m0 + mi * 32 + ln;
    if (m >= M) continue;
    size_t pbase = 0;
    int tok = 0;
    if (head >= Hq) {                                 // k or v head: locate the row's cache slot
      const int b = p.row_seq[m];
      const int pos = p.seq_c[b] + p.row_pos[m];
      const int page = kv.block_table[(size_t)p.seq_slot[b] * kv.max_pages + pos / kPage];
      tok = pos % kPage;
      pbase = (size_t)page * kv_page_elems(Hkv, kD);
    }
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int d = 32 * wave + 8 * i4 + 4 * lg;      // four consecutive head columns d .. d + 3
      float y[4];
      if (is_v) {
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = acc[mi][0][4 * i4 + e];
      } else {
        const int j = d & 63;
        const f32x4 c = *(const f32x4*)(cos_t + (size_t)m * 64 + j), sn = *(const f32x4*)(sin_t + (size_t)m * 64 + j);
        const f32x4 other = *(const f32x4*)(s_x + (mi * 32 + ln) * LDX + d + partner);
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = acc[mi][0][4 * i4 + e] * c[e] + sign * other[e] * sn[e];
      }
      if (head < Hq) {
        *(f16x4*)(q_out + ((size_t)m * Hq + head) * kD + d) = to_f16x4_guarded(y[0], y[1], y[2], y[3], p.status);
      } else {
        // bf16-rounded values in float16 encoding (page format)
        const f16x4 v = to_f16x4_guarded((float)(bf16)y[0], (float)(bf16)y[1], (float)(bf16)y[2], (float)(bf16)y[3], p.status);
        if (!is_v) {
          *(f16x4*)(k_pages + pbase + k_index_bf16(kD, head - Hq, tok, d)) = v;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) v_pages[pbase + v_index_bf16(kD, head - Hq - Hkv, tok, d + e)] = v[e];
        }
      }
    }
  }
}

template <int MT>
void launch_t(const Shape& s, const Plan& p, const KvView& kv, int M_max, const void* A, const void* Wp,
              const float* cos_t, const float* sin_t, void* q_out, void* k_pages, void* v_pages, hipStream_t st) {
  using G = MfmaGemm<MT, 1, true>;
  const int m_blocks = (M_max + G::BM - 1) / G::BM, heads = s.Hq + 2 * s.Hkv;
  size_t lds = G::LDS_BYTES;
  const size_t lds_x = (size_t)32 * MT * (kD + 4) * 4;
  if (lds < lds_x) lds = lds_x;
  static bool attr_set = false;
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)qkv_rope_kernel<MT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr_set = true; }
  const int grid = 8 * ((m_blocks * heads + 7) / 8);
  hipLaunchKernelGGL((qkv_rope_kernel<MT>), dim3(grid), dim3(256), lds, st, p, kv, M_max, s.d, s.Hq, s.Hkv,
                     (const f16*)A, (const f16*)Wp, cos_t, sin_t, (f16*)q_out, (f16*)k_pages, (f16*)v_pages, m_blocks,
                     m_blocks * heads <= 512 ? 1 : 0);
}
}  // namespace

bool qkv_rope_supported(const Shape& s) { return s.dtype == BS_BF16 && s.D == kD; }

void launch_qkv_rope(const Shape& s, const Plan& p, const KvView& kv, int M_max, const void* A, const void* Wp,
                     const float* cos_t, const float* sin_t, void* q_out, void* k_pages, void* v_pages, hipStream_t st) {
  // 32-row tiles while that gives at most two workgroups per CU (measured at M = 576, 16 heads: 13.5 us
  // against 15.3 us with 64-row tiles); larger tiles re-read the weights less often when there are many rows
  const int tiles1 = (M_max + 31) / 32 * (s.Hq + 2 * s.Hkv);
  int mt = tiles1 <= 512 ? 1 : (tiles1 <= 2048 ? 2 : 4);
  // between one and two 32-row workgroups per CU with a long contraction, 64-row tiles (at most one workgroup per
  // CU, half the weight re-reads) are faster: 7B shape, 288 rows x 36 heads, 42.5 -> 33.4 us; with the short
  // contraction of the 1.5B shape (576 rows x 16 heads) they are not: 20.3 -> 21.8 us
  if (tiles1 > 256 && tiles1 <= 512 && s.d >= 2048) mt = 2;
  if (mt <= 1) launch_t<1>(s, p, kv, M_max, A, Wp, cos_t, sin_t, q_out, k_pages, v_pages, st);
  else if (mt == 2) launch_t<2>(s, p, kv, M_max, A, Wp, cos_t, sin_t, q_out, k_pages, v_pages, st);
  else launch_t<4>(s, p, kv, M_max, A, Wp, cos_t, sin_t, q_out, k_pages, v_pages, st);
}
