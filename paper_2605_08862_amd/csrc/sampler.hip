// LM head fused with softmax statistics, the accept scan of Alg. 1 and the residual / bonus
// sampling of Eq. 2-3.  The [M, V] probabilities are never formed in HBM:
//   phase 1  LM-head GEMM over all M rows whose epilogue keeps, per (row, vocabulary tile), only
//            (max, sum exp, arg max) of z/T and the logit of the draft token judged by the row;
//   scan     per sequence, the first rejected draft (Eq. 2, general form min(1, p/q));
//   phase 2  the one row per sequence that is sampled from (recovered, bonus or plain token) is
//            recomputed by the same MFMA loop (bit-identical logits) and sampled by inverse CDF in
//            vocabulary order with float64 running sums (Eq. 3 / max(0, p - q)).
#include "gemm_mfma.h"

enum { MODE_NONE = 0, MODE_PLAIN = 1, MODE_RESID_ONEHOT = 2, MODE_RESID_DENSE = 3 };

constexpr int kLmNT = 2;                            // LM-head wave tile: 32*MT rows x 64 vocab entries
constexpr int kLmVtile = kLmNT * 32;                // vocab entries per statistics tile (bf16 path)
constexpr int kSampleChunks = 32;                   // vocabulary chunks per sequence in the sampling kernels
constexpr int kRowVtile = 1024;                     // vocab entries per statistics tile (logits path)

int lmhead_vtiles(int V) {
  int a = (V + kLmVtile - 1) / kLmVtile, b = (V + kRowVtile - 1) / kRowVtile;
  return a > b ? a : b;
}

// ------------------------------------------------------------------ phase 1 / phase 2 GEMM (bf16)
// STATS = true : rows are the packed query rows; epilogue writes statistics (+ optional debug logits).
// STATS = false: rows are gathered through sel_row (one per sequence); epilogue stores float32 logits
//                to sel_logits [B, V].
template <int kLmMT, bool STATS>
__global__ void __launch_bounds__(256, (kLmMT <= 3 ? 2 : 1)) lmhead_kernel(const int32_t* __restrict__ n_rows_dev, int M_max, int V, int K,
                                                     const f16* __restrict__ X, const int32_t* __restrict__ x_rows,
                                                     const f16* __restrict__ W, float inv_temp,
                                                     const int32_t* __restrict__ row_target, SamplerBufs sb,
                                                     float* __restrict__ store, int m_blocks, int n_blocks) {
  using G = MfmaGemm<kLmMT, kLmNT, true>;
  extern __shared__ __align__(16) char lds[];
  const int M = n_rows_dev ? min(*n_rows_dev, M_max) : M_max;
  const int total = m_blocks * n_blocks;
  const int per_xcd = (total + 7) / 8;
  const int id = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (id >= total) return;
  const int mb = id % m_blocks, nb = id / m_blocks;
  const int m0 = mb * G::BM;
  if (m0 >= M) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int vt = nb * 4 + wave;                       // statistics tile of this wave
  const int n_wave0 = vt * kLmVtile;

  typename G::Operands op;
#pragma unroll
  for (int i = 0; i < kLmMT; ++i) {
    int row, g, s;
    G::chunk_of(i, row, g, s);
    int r = min(m0 + row, M - 1);
    if (x_rows) r = x_rows[r];
    op.x_rows[i] = X + (size_t)r * K + g * 32 + s * 8;
    op.x_lds[i] = G::chunk_lds_offset(row, g, s);
  }
  const int nk = K / kBK;
  const int n_tiles = (V + 31) / 32;
#pragma unroll
  for (int ni = 0; ni < kLmNT; ++ni) {
    const int nt = min(n_wave0 / 32 + ni, n_tiles - 1);
    op.w_tiles[ni] = W + (size_t)nt * nk * kWBlock + lane * 8;
  }
  f32x16 acc[kLmMT][kLmNT];
#pragma unroll
  for (int mi = 0; mi < kLmMT; ++mi)
#pragma unroll
    for (int ni = 0; ni < kLmNT; ++ni)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.f;
  G::run(acc, op, 0, nk, lds);
  if (n_wave0 >= V) return;

  // accumulator (SWAP): rows = vocabulary entries n_wave0 + ni*32 + acc_row, lane column = token
  const bool store_vec = (V & 3) == 0 && ((uintptr_t)store & 15) == 0;   // V % 4 == 0: groups of four never straddle V
#pragma unroll
  for (int mi = 0; mi < kLmMT; ++mi) {
    const int m = m0 + mi * 32 + acc_col(lane);
    const bool valid = m < M;
    if (STATS) {
      const int tgt = valid ? row_target[m] : -1;
      float mx = -INFINITY, zt = 0.f;
      int arg = 0x7fffffff;
      bool hit = false;
      // no store inside this loop: the draft token's logit is picked up by a select (a conditional store at each of
      // the 32 positions cost 13 us of the 277 us launch)
#pragma unroll
      for (int ni = 0; ni < kLmNT; ++ni)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int n = n_wave0 + ni * 32 + acc_row(lane, i);
          const float z = acc[mi][ni][i];
          if (n < V) {
            if (z > mx) { mx = z; arg = n; }
            if (n == tgt) { zt = z; hit = true; }
          }
        }
      if (hit) sb.z_target[m] = zt;                    // tgt >= 0 only for valid rows
      if (valid && store && !store_vec) {
#pragma unroll
        for (int ni = 0; ni < kLmNT; ++ni)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int n = n_wave0 + ni * 32 + acc_row(lane, i);
            if (n < V) store[(size_t)m * V + n] = acc[mi][ni][i];
          }
      }
      if (valid && store && store_vec) {
        // registers 4 i4 .. 4 i4 + 3 of a lane are four consecutive vocabulary entries: 16-byte stores
#pragma unroll
        for (int ni = 0; ni < kLmNT; ++ni)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const int n = n_wave0 + ni * 32 + acc_row(lane, 4 * i4);
            if (n + 3 < V)
              *(f32x4*)(store + (size_t)m * V + n) =
                  f32x4{acc[mi][ni][4 * i4], acc[mi][ni][4 * i4 + 1], acc[mi][ni][4 * i4 + 2], acc[mi][ni][4 * i4 + 3]};
          }
      }
      const float mx_o = __shfl_xor(mx, 32);
      const int arg_o = __shfl_xor(arg, 32);
      if (mx_o > mx || (mx_o == mx && arg_o < arg)) { mx = mx_o; arg = arg_o; }
      float sum = 0.f;
#pragma unroll
      for (int ni = 0; ni < kLmNT; ++ni)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int n = n_wave0 + ni * 32 + acc_row(lane, i);
          if (n < V) sum += __expf((acc[mi][ni][i] - mx) * inv_temp);
        }
      sum += __shfl_xor(sum, 32);
      if (valid && lane < 32) {
        const size_t o = (size_t)vt * M_max + m;
        sb.part_max[o] = mx;
        sb.part_sum[o] = sum;
        sb.part_arg[o] = arg;
      }
    } else {
      if (!valid) continue;
      // registers 4 i4 .. 4 i4 + 3 of a lane are four consecutive vocabulary entries: 16-byte stores when the
      // row pitch keeps them aligned
      const bool vec = (V & 3) == 0;
#pragma unroll
      for (int ni = 0; ni < kLmNT; ++ni)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const int n = n_wave0 + ni * 32 + acc_row(lane, 4 * i4);
          if (vec && n + 3 < V) {
            *(f32x4*)(store + (size_t)m * V + n) =
                f32x4{acc[mi][ni][4 * i4], acc[mi][ni][4 * i4 + 1], acc[mi][ni][4 * i4 + 2], acc[mi][ni][4 * i4 + 3]};
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n + e < V) store[(size_t)m * V + n + e] = acc[mi][ni][4 * i4 + e];
          }
        }
    }
  }
}

// ------------------------------------------------------------------ statistics of given float32 logits
__global__ void __launch_bounds__(256) logit_stats_kernel(Plan p, int M_max, int V, const float* __restrict__ logits,
                                                          float inv_temp, SamplerBufs sb) {
  __shared__ float s_mx[4], s_sum[4];
  __shared__ int s_arg[4];
  const int m = blockIdx.y, vt = blockIdx.x;
  if (m >= p.n_rows[0]) return;
  const int tgt = p.row_target[m];
  const float* z = logits + (size_t)m * V;
  const int base = vt * kRowVtile;
  float v[4];
  float mx = -INFINITY;
  int arg = 0x7fffffff;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int n = base + j * 256 + threadIdx.x;
    v[j] = (n < V) ? z[n] : -INFINITY;
    if (n < V && n == tgt) sb.z_target[m] = v[j];
    if (v[j] > mx) { mx = v[j]; arg = n; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    float mo = __shfl_xor(mx, o);
    int ao = __shfl_xor(arg, o);
    if (mo > mx || (mo == mx && ao < arg)) { mx = mo; arg = ao; }
  }
  if ((threadIdx.x & 63) == 0) { s_mx[threadIdx.x >> 6] = mx; s_arg[threadIdx.x >> 6] = arg; }
  __syncthreads();
  mx = s_mx[0]; arg = s_arg[0];
  for (int w = 1; w < 4; ++w)
    if (s_mx[w] > mx || (s_mx[w] == mx && s_arg[w] < arg)) { mx = s_mx[w]; arg = s_arg[w]; }
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) sum += (v[j] == -INFINITY) ? 0.f : __expf((v[j] - mx) * inv_temp);
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if ((threadIdx.x & 63) == 0) s_sum[threadIdx.x >> 6] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    const size_t o = (size_t)vt * M_max + m;
    sb.part_max[o] = mx;
    sb.part_sum[o] = s_sum[0] + s_sum[1] + s_sum[2] + s_sum[3];
    sb.part_arg[o] = arg;
  }
}

// ------------------------------------------------------------------ per-row statistics
// Stage 1 folds the per-tile (max, sum exp, arg max) entries of 32 consecutive rows over one of kStatChunks
// ranges of vocabulary tiles into one entry per (row, range) with the same meaning.  Tile entries of a row
// are M_max apart, so a workgroup reads 32 rows x 8 tiles at a time: every 128-byte line it touches is used
// completely (one workgroup per row touched a new line for every 4-byte entry: 175 MB fetched for 16 MB).
constexpr int kStatChunks = 16;
__global__ void __launch_bounds__(256) row_stats_fold_kernel(Plan p, int M_max, int n_vtiles, float inv_temp, SamplerBufs sb) {
  __shared__ float s_mx[8][32], s_sum[8][32];
  __shared__ int s_arg[8][32];
  const int rr = threadIdx.x & 31, vl = threadIdx.x >> 5;
  const int r = blockIdx.x * 32 + rr, ch = blockIdx.y;
  const int per = (n_vtiles + kStatChunks - 1) / kStatChunks;
  const int v0 = min(ch * per, n_vtiles), v1 = min(v0 + per, n_vtiles);
  const bool valid = r < min(p.n_rows[0], M_max);
  float mx = -INFINITY, sum = 0.f;
  int arg = 0x7fffffff;
  auto fold = [&](float m2, float s2, int a2) {
    if (m2 > mx) { sum = sum * __expf((mx - m2) * inv_temp) + s2; mx = m2; arg = a2; }
    else if (m2 > -INFINITY) { sum += s2 * __expf((m2 - mx) * inv_temp); if (m2 == mx && a2 < arg) arg = a2; }
  };
  if (valid) {
    // four tile entries are requested before the first is folded (same order of folding): one memory round trip
    // per four entries instead of one per entry
    int vt = v0 + vl;
    for (; vt + 24 < v1; vt += 32) {
      float m4[4], s4[4];
      int a4[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const size_t o = (size_t)(vt + 8 * u) * M_max + r;
        m4[u] = sb.part_max[o]; s4[u] = sb.part_sum[o]; a4[u] = sb.part_arg[o];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) fold(m4[u], s4[u], a4[u]);
    }
    for (; vt < v1; vt += 8) {
      const size_t o = (size_t)vt * M_max + r;
      fold(sb.part_max[o], sb.part_sum[o], sb.part_arg[o]);
    }
  }
  s_mx[vl][rr] = mx; s_sum[vl][rr] = sum; s_arg[vl][rr] = arg;
  __syncthreads();
  if (vl == 0 && valid) {
    for (int w = 1; w < 8; ++w) fold(s_mx[w][rr], s_sum[w][rr], s_arg[w][rr]);
    const size_t o = (size_t)ch * M_max + r;
    sb.fold_max[o] = mx; sb.fold_sum[o] = sum; sb.fold_arg[o] = arg;
  }
}

// Stage 2 (also the only stage for the few 1024-entry tiles of the plain-logits path):
__global__ void __launch_bounds__(256) row_stats_kernel(Plan p, int M_max, int n_vtiles, float inv_temp, SamplerBufs sb,
                                                        const float* __restrict__ t_max, const float* __restrict__ t_sum,
                                                        const int32_t* __restrict__ t_arg) {
  __shared__ float s_mx[4], s_sum[4];
  __shared__ int s_arg[4];
  const int r = blockIdx.x, tid = threadIdx.x;
  if (r >= p.n_rows[0]) return;
  float mx = -INFINITY;
  int arg = 0x7fffffff;
  for (int vt = tid; vt < n_vtiles; vt += 256) {
    const float m2 = t_max[(size_t)vt * M_max + r];
    const int a2 = t_arg[(size_t)vt * M_max + r];
    if (m2 > mx || (m2 == mx && a2 < arg)) { mx = m2; arg = a2; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    const float mo = __shfl_xor(mx, o);
    const int ao = __shfl_xor(arg, o);
    if (mo > mx || (mo == mx && ao < arg)) { mx = mo; arg = ao; }
  }
  if ((tid & 63) == 0) { s_mx[tid >> 6] = mx; s_arg[tid >> 6] = arg; }
  __syncthreads();
  mx = s_mx[0]; arg = s_arg[0];
  for (int w = 1; w < 4; ++w)
    if (s_mx[w] > mx || (s_mx[w] == mx && s_arg[w] < arg)) { mx = s_mx[w]; arg = s_arg[w]; }
  float sum = 0.f;
  for (int vt = tid; vt < n_vtiles; vt += 256) {
    const float m2 = t_max[(size_t)vt * M_max + r];
    if (m2 > -INFINITY) sum += t_sum[(size_t)vt * M_max + r] * __expf((m2 - mx) * inv_temp);
  }
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if ((tid & 63) == 0) s_sum[tid >> 6] = sum;
  __syncthreads();
  if (tid == 0) {
    sb.row_max[r] = mx;
    sb.row_lse[r] = mx * inv_temp + logf(s_sum[0] + s_sum[1] + s_sum[2] + s_sum[3]);
    sb.row_arg[r] = arg;
  }
}

// ------------------------------------------------------------------ proposal statistics
// For every query row that judges a draft: max and log-sum-exp of its q_logits row and q_logits[draft].
// One pass (online max / rescaled sum), 16-byte loads.
template <typename Q> struct QVec;
template <> struct QVec<float> { static constexpr int N = 4; };
template <> struct QVec<bf16> { static constexpr int N = 8; };

template <typename Q>
__global__ void __launch_bounds__(256) q_stats_kernel(Plan p, int V, const Q* __restrict__ q_logits, SamplerBufs sb) {
  __shared__ float s_m[4], s_s[4];
  const int r = blockIdx.x, tid = threadIdx.x;
  if (r >= p.n_rows[0]) return;
  const int tgt = p.row_target[r];
  if (tgt < 0) return;
  const int b = p.row_seq[r];
  const Q* q = q_logits + (size_t)(p.draft_start[b] + p.row_pos[r]) * V;
  constexpr int N = QVec<Q>::N;
  float m = -INFINITY, sum = 0.f;
  auto absorb = [&](float x) {
    if (x > m) { sum = sum * __expf(m - x) + 1.0f; m = x; }   // exp(-inf) = 0 on the first element
    else sum += __expf(x - m);
  };
  // one 16-byte vector: a single rescale for its maximum, then N exponentials
  auto absorb_vec = [&](const u32x4 raw) {
    float x[N];
    if (N == 4) {
#pragma unroll
      for (int j = 0; j < 4; ++j) x[j] = __uint_as_float(raw[j]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) { x[2 * j] = __uint_as_float(raw[j] << 16); x[2 * j + 1] = __uint_as_float(raw[j] & 0xffff0000u); }
    }
    float vm = x[0];
#pragma unroll
    for (int j = 1; j < N; ++j) vm = fmaxf(vm, x[j]);
    if (vm == -INFINITY) return;
    if (vm > m) { sum *= __expf(m - vm); m = vm; }
#pragma unroll
    for (int j = 0; j < N; ++j) sum += __expf(x[j] - m);
  };
  const bool aligned = (((uintptr_t)q) & 15) == 0;
  const int nvec = aligned ? V / N : 0;
  int i = tid;
  for (; i + 7 * 256 < nvec; i += 8 * 256) {           // eight vectors in flight per thread: with one workgroup per
    u32x4 r[8];                                        // row (two per CU) the bytes in flight, not HBM, set the rate
#pragma unroll
    for (int u = 0; u < 8; ++u) r[u] = *(const u32x4*)(q + (size_t)(i + u * 256) * N);
#pragma unroll
    for (int u = 0; u < 8; ++u) absorb_vec(r[u]);
  }
  for (; i < nvec; i += 256) absorb_vec(*(const u32x4*)(q + (size_t)i * N));
  for (int n = nvec * N + tid; n < V; n += 256) absorb(to_f32<Q>(q[n]));
  for (int o = 32; o > 0; o >>= 1) {
    const float mo = __shfl_xor(m, o), so = __shfl_xor(sum, o);
    const float mn = fmaxf(m, mo);
    sum = (m == -INFINITY ? 0.f : sum * __expf(m - mn)) + (mo == -INFINITY ? 0.f : so * __expf(mo - mn));
    m = mn;
  }
  if ((tid & 63) == 0) { s_m[tid >> 6] = m; s_s[tid >> 6] = sum; }
  __syncthreads();
  if (tid == 0) {
    float mt = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3])), st = 0.f;
    for (int w = 0; w < 4; ++w) if (s_m[w] > -INFINITY) st += s_s[w] * __expf(s_m[w] - mt);
    sb.q_max[r] = mt;
    sb.q_lse[r] = mt + logf(st);
    sb.q_target[r] = to_f32<Q>(q[tgt]);
  }
}

// ------------------------------------------------------------------ accept scan (Alg. 1 inner loop, Eq. 2)
// One thread per sequence: the first rejected draft, the row that will be sampled from and how.
__global__ void __launch_bounds__(64) accept_scan_kernel(Plan p, int B, int k_max, int dense_q, float temperature,
                                                         int eos_id, int emit_bonus, int filter_on,
                                                         const float* __restrict__ u_accept,
                                                         SamplerBufs sb, int32_t* __restrict__ n_accepted,
                                                         int32_t* __restrict__ out_tokens, int32_t* __restrict__ n_emitted,
                                                         uint32_t* __restrict__ near_tie) {
  const int b = blockIdx.x * 64 + threadIdx.x;
  if (b >= B) return;
  const int k = p.seq_k[b];
  int32_t* out = out_tokens + (size_t)b * (k_max + 1);
  if (k < 0) {                                      // sequence skipped by the plan
    n_accepted[b] = 0; n_emitted[b] = 0; near_tie[b] = 0; sb.sel_mode[b] = MODE_NONE; sb.sel_row[b] = 0;
    for (int i = 0; i <= k_max; ++i) out[i] = -1;
    return;
  }
  const int r0 = p.row_start[b];
  const float inv_temp = temperature > 0.f ? 1.0f / temperature : 1.0f;
  int n_acc = 0, mode = MODE_NONE, sel = r0, sel_tok = -1, n_out = 0;
  uint32_t tie = 0;
  bool stopped = false, eos = false;
  for (int i = 0; i < k && !stopped; ++i) {
    const int r = r0 + i;
    const int x = p.row_target[r];
    float px;
    if (temperature > 0.f && filter_on)             // filtered target: zero outside the kept set, renormalised inside
      px = filter_keeps(filter_key(sb.z_target[r]), x, sb.f_key[r], sb.f_idx[r])
               ? __expf(sb.z_target[r] * inv_temp - sb.f_lse[r]) : 0.0f;
    else if (temperature > 0.f) px = __expf(sb.z_target[r] * inv_temp - sb.row_lse[r]);
    else px = (x == sb.row_arg[r]) ? 1.0f : 0.0f;
    float rho = px;
    if (dense_q) {
      const float qx = __expf(sb.q_target[r] - sb.q_lse[r]);
      rho = (qx == 0.f) ? INFINITY : px / qx;
    }
    const float u = u_accept[(size_t)b * k_max + i];
    if (fabsf(rho - u) <= 1e-3f) tie |= 1u << i;
    if (u < fminf(1.0f, rho)) {
      out[n_out++] = x;
      ++n_acc;
      if (x == eos_id) { stopped = true; eos = true; }
    } else {
      sel = r; sel_tok = x;
      mode = dense_q ? MODE_RESID_DENSE : MODE_RESID_ONEHOT;
      stopped = true;
    }
  }
  if (mode == MODE_NONE && !eos && (emit_bonus || k == 0)) {
    sel = r0 + k;
    mode = MODE_PLAIN;
  }
  if (mode != MODE_NONE && temperature == 0.f) {    // one-hot target: every sampled token is the arg-max
    out[n_out++] = sb.row_arg[sel];
    mode = MODE_NONE;
  }
  for (int i = n_out; i <= k_max; ++i) out[i] = -1;
  n_accepted[b] = n_acc;
  n_emitted[b] = n_out;
  near_tie[b] = tie;
  sb.sel_row[b] = sel;
  sb.sel_mode[b] = mode;
  sb.sel_tok[b] = sel_tok;
  sb.sel_qrow[b] = p.draft_start[b] + (sel - r0);
  sb.sel_pmax[b] = sb.row_max[sel];
  sb.sel_qmax[b] = (mode == MODE_RESID_DENSE) ? sb.q_max[sel] : 0.f;
}

// ------------------------------------------------------------------ inverse-CDF sampling (Eq. 3)
// The vocabulary of each sampled row is cut into kSampleChunks chunks so that B x 32 workgroups share
// the float64 exponentials.  Three small kernels: normaliser partials, chunk masses, pick.
//   p_j = exp(z_j/T - max) / sum_p ;  q_j likewise ;  w_j = p_j | p_j [j != draft] | max(0, p_j - q_j)
// Divisions by per-row constants (T, the two normalisers) are multiplications by their float64 reciprocals: a
// float64 division costs about as much as the exponential next to it, and the one-ulp difference is far below
// what the order of the running sums already leaves open.
template <typename Q, bool FILT>
struct SampleRow {
  const float* z; const Q* q; double inv_T, mxp, mxq; int tgt, mode;
  int f_idx; uint32_t f_key;                         // top-k / top-p threshold of the row (FILT only)
  // the *_v forms take the logits as values (callers that request many loads before using the first)
  __device__ double e_p_v(int j, float zj) const {
    if (FILT && !filter_keeps(filter_key(zj), j, f_key, f_idx)) return 0.0;
    return exp((double)zj * inv_T - mxp);
  }
  __device__ double e_q_v(float qj) const { return exp((double)qj - mxq); }
  __device__ double e_p(int j) const { return e_p_v(j, z[j]); }
  __device__ double e_q(int j) const { return e_q_v(to_f32<Q>(q[j])); }
  // inv_sp, inv_sq: reciprocals of the normalisers
  __device__ double weight_v(int j, float zj, float qj, double inv_sp, double inv_sq, int mode_now) const {
    const double pj = e_p_v(j, zj) * inv_sp;
    if (mode_now == MODE_PLAIN) return pj;
    if (mode_now == MODE_RESID_ONEHOT) return j == tgt ? 0.0 : pj;
    return fmax(0.0, pj - e_q_v(qj) * inv_sq);
  }
  __device__ double weight(int j, double inv_sp, double inv_sq, int mode_now) const {
    return weight_v(j, z[j], (mode_now == MODE_RESID_DENSE) ? to_f32<Q>(q[j]) : 0.f, inv_sp, inv_sq, mode_now);
  }
};

template <typename Q, bool FILT>
__device__ __forceinline__ SampleRow<Q, FILT> sample_row(int b, int V, const float* logit_base, int rows_are_selected,
                                                         const Q* q_logits, float temperature, const SamplerBufs& sb) {
  SampleRow<Q, FILT> r;
  r.mode = sb.sel_mode[b];
  r.f_key = FILT ? sb.f_key[sb.sel_row[b]] : 0u;
  r.f_idx = FILT ? sb.f_idx[sb.sel_row[b]] : 0;
  r.z = logit_base + (size_t)(rows_are_selected ? b : sb.sel_row[b]) * V;
  r.q = (r.mode == MODE_RESID_DENSE) ? q_logits + (size_t)sb.sel_qrow[b] * V : nullptr;
  r.inv_T = 1.0 / (double)temperature;
  r.mxp = (double)sb.sel_pmax[b] * r.inv_T;          // max_j z_j/T: the scaling is monotone
  r.mxq = (double)sb.sel_qmax[b];
  r.tgt = sb.sel_tok[b];
  return r;
}

__device__ __forceinline__ double block_sum_f64(double v, double* red) {     // 256 threads
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

template <typename Q, bool FILT>
__global__ void __launch_bounds__(256) sample_sum_kernel(int V, const float* __restrict__ logit_base, int rows_are_selected,
                                                         const Q* __restrict__ q_logits, float temperature, SamplerBufs sb) {
  __shared__ double red[4];
  const int c = blockIdx.x, b = blockIdx.y;
  if (sb.sel_mode[b] == MODE_NONE) return;
  const SampleRow<Q, FILT> r = sample_row<Q, FILT>(b, V, logit_base, rows_are_selected, q_logits, temperature, sb);
  const int chunk = (V + kSampleChunks - 1) / kSampleChunks;
  const int j0 = min(c * chunk, V), j1 = min(j0 + chunk, V);
  double sp = 0.0, sq = 0.0;
  for (int j = j0 + threadIdx.x; j < j1; j += 256) {
    sp += r.e_p(j);
    if (r.q) sq += r.e_q(j);
  }
  sp = block_sum_f64(sp, red);
  sq = block_sum_f64(sq, red);
  if (threadIdx.x == 0) {
    sb.samp_sum[((size_t)b * kSampleChunks + c) * 2] = sp;
    sb.samp_sum[((size_t)b * kSampleChunks + c) * 2 + 1] = sq;
  }
}

// Reciprocals of the two normalisers of sequence b (0 for an absent proposal).
__device__ __forceinline__ void sample_totals(const SamplerBufs& sb, int b, double& inv_sp, double& inv_sq) {
  double sp = 0.0, sq = 0.0;
  for (int c = 0; c < kSampleChunks; ++c) {          // fixed order: every workgroup gets the same totals
    sp += sb.samp_sum[((size_t)b * kSampleChunks + c) * 2];
    sq += sb.samp_sum[((size_t)b * kSampleChunks + c) * 2 + 1];
  }
  inv_sp = 1.0 / sp;
  inv_sq = sq > 0.0 ? 1.0 / sq : 0.0;
}

// chunk masses of the residual (index 0) and of p itself (index 1, used when the residual is empty)
template <typename Q, bool FILT>
__global__ void __launch_bounds__(256) sample_mass_kernel(int V, const float* __restrict__ logit_base, int rows_are_selected,
                                                          const Q* __restrict__ q_logits, float temperature, SamplerBufs sb) {
  __shared__ double red[4];
  const int c = blockIdx.x, b = blockIdx.y;
  if (sb.sel_mode[b] == MODE_NONE) return;
  const SampleRow<Q, FILT> r = sample_row<Q, FILT>(b, V, logit_base, rows_are_selected, q_logits, temperature, sb);
  double sp, sq;
  sample_totals(sb, b, sp, sq);
  const int chunk = (V + kSampleChunks - 1) / kSampleChunks;
  const int j0 = min(c * chunk, V), j1 = min(j0 + chunk, V);
  double mw = 0.0, mp = 0.0;
  for (int j = j0 + threadIdx.x; j < j1; j += 256) {
    mw += r.weight(j, sp, sq, r.mode);
    mp += r.e_p(j) * sp;
  }
  mw = block_sum_f64(mw, red);
  mp = block_sum_f64(mp, red);
  if (threadIdx.x == 0) {
    sb.samp_mass[((size_t)b * kSampleChunks + c) * 2] = mw;
    sb.samp_mass[((size_t)b * kSampleChunks + c) * 2 + 1] = mp;
  }
}

constexpr int kPickThreads = 1024;
template <typename Q, bool FILT>
__global__ void __launch_bounds__(kPickThreads) sample_pick_kernel(int V, const float* __restrict__ logit_base, int rows_are_selected,
                                                          const Q* __restrict__ q_logits, float temperature,
                                                          const float* __restrict__ u_sample, SamplerBufs sb,
                                                          const int32_t* __restrict__ n_accepted, int k_max,
                                                          int32_t* __restrict__ out_tokens, int32_t* __restrict__ n_emitted,
                                                          uint32_t* __restrict__ near_tie) {
  __shared__ double s_scan[kPickThreads];
  __shared__ int s_i[2];
  const int b = blockIdx.x, tid = threadIdx.x;
  if (sb.sel_mode[b] == MODE_NONE) return;
  const SampleRow<Q, FILT> r = sample_row<Q, FILT>(b, V, logit_base, rows_are_selected, q_logits, temperature, sb);
  double sp, sq;
  sample_totals(sb, b, sp, sq);
  // chunk level (every thread walks the 32 chunk masses: same result in all threads)
  int mode = r.mode;
  double total = 0.0;
  for (int c = 0; c < kSampleChunks; ++c) total += sb.samp_mass[((size_t)b * kSampleChunks + c) * 2];
  if (!(total > 0.0) && mode != MODE_PLAIN) {       // empty residual: fall back to the target itself
    mode = MODE_PLAIN;
    total = 0.0;
    for (int c = 0; c < kSampleChunks; ++c) total += sb.samp_mass[((size_t)b * kSampleChunks + c) * 2 + 1];
  }
  const int mi = (mode == r.mode) ? 0 : 1;
  const double t = (double)u_sample[b] * total;
  int cs = -1, last_c = -1;
  double excl_c = 0.0, run = 0.0, last_excl = 0.0;
  for (int c = 0; c < kSampleChunks; ++c) {
    const double m = sb.samp_mass[((size_t)b * kSampleChunks + c) * 2 + mi];
    if (m > 0.0) { last_c = c; last_excl = run; }
    if (cs < 0 && run + m > t) { cs = c; excl_c = run; }
    run += m;
  }
  if (cs < 0) { cs = last_c; excl_c = last_excl; }  // rounding left no chunk: last chunk with weight
  if (cs < 0) return;                               // no weight anywhere (cannot happen for finite logits)
  // slice level inside the chosen chunk
  const int chunk = (V + kSampleChunks - 1) / kSampleChunks;
  const int c0 = min(cs * chunk, V), c1 = min(c0 + chunk, V);
  const int slice = (c1 - c0 + kPickThreads - 1) / kPickThreads;
  const int j0 = min(c0 + tid * slice, c1), j1 = min(j0 + slice, c1);
  // One workgroup per sequence: nothing hides a load's latency here, so a thread requests its whole slice (up to
  // kW logits of p and q) at once and keeps the weights in registers for the walk below.  1024 threads: the two
  // float64 exponentials per token are the bulk of this kernel and only B workgroups share the GPU.
  constexpr int kW = 8;
  const bool in_regs = slice <= kW;
  double wv[kW];
  double csum = 0.0;
  if (in_regs) {
    float zr[kW], qr[kW];
#pragma unroll
    for (int i = 0; i < kW; ++i) {
      const int jj = min(j0 + i, V - 1);
      zr[i] = r.z[jj];
      qr[i] = (mode == MODE_RESID_DENSE) ? to_f32<Q>(r.q[jj]) : 0.f;
    }
#pragma unroll
    for (int i = 0; i < kW; ++i) {
      wv[i] = 0.0;
      if (j0 + i < j1) wv[i] = r.weight_v(j0 + i, zr[i], qr[i], sp, sq, mode);
      csum += wv[i];
    }
  } else {
    for (int j = j0; j < j1; ++j) csum += r.weight(j, sp, sq, mode);
  }
  s_scan[tid] = csum;
  __syncthreads();
  for (int o = 1; o < kPickThreads; o <<= 1) {
    const double v = (tid >= o) ? s_scan[tid - o] : 0.0;
    __syncthreads();
    s_scan[tid] += v;
    __syncthreads();
  }
  const double incl = excl_c + s_scan[tid], excl = incl - csum;
  if (tid == 0) { s_i[0] = 0x7fffffff; s_i[1] = -1; }
  __syncthreads();
  if (csum > 0.0) {
    if (incl > t && excl <= t) atomicMin(&s_i[0], tid);
    atomicMax(&s_i[1], tid);
  }
  __syncthreads();
  const int owner = (s_i[0] != 0x7fffffff) ? s_i[0] : s_i[1];
  if (tid != owner) return;
  double acc = excl, w = 0.0, last_hi = 0.0, last_w = 0.0;
  int tok = -1, last = -1;
  if (in_regs) {
    bool found = false;
#pragma unroll
    for (int i = 0; i < kW; ++i) {
      const int j = j0 + i;
      if (!found && j < j1) {
        w = wv[i];
        acc += w;
        if (w > 0.0) { last = j; last_hi = acc; last_w = w; }
        if (acc > t) { tok = j; found = true; }
      }
    }
  } else {
    for (int j = j0; j < j1; ++j) {
      w = r.weight(j, sp, sq, mode);
      acc += w;
      if (w > 0.0) { last = j; last_hi = acc; last_w = w; }
      if (acc > t) { tok = j; break; }
    }
  }
  if (tok < 0) { tok = last; acc = last_hi; w = last_w; }
  const int n_acc = n_accepted[b];
  out_tokens[(size_t)b * (k_max + 1) + n_acc] = tok;
  n_emitted[b] = n_acc + 1;
  const double lo = acc - w;
  if (fmin(fabs(t - lo), fabs(acc - t)) <= 1e-3 * w) near_tie[b] |= 0x80000000u;
}

// ------------------------------------------------------------------ launchers
template <int MT, bool STATS>
static void launch_lmhead_t(const Shape& s, const int32_t* n_rows_dev, int M_max, const void* hf, const int32_t* x_rows,
                            const void* lm_head, float inv_temp, const int32_t* row_target, const SamplerBufs& sb,
                            float* store, hipStream_t st) {
  using G = MfmaGemm<MT, kLmNT, true>;
  int m_blocks = (M_max + G::BM - 1) / G::BM, n_blocks = (s.V + 4 * kLmVtile - 1) / (4 * kLmVtile);
  int grid = ((m_blocks * n_blocks + 7) / 8) * 8;
  static bool attr_set = false;              // more than 64 KiB of dynamic LDS needs an opt-in (192-row tiles)
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)lmhead_kernel<MT, STATS>, hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES); attr_set = true; }
  hipLaunchKernelGGL((lmhead_kernel<MT, STATS>), dim3(grid), dim3(256), G::LDS_BYTES, st, n_rows_dev, M_max, s.V, s.d,
                     (const f16*)hf, x_rows, (const f16*)lm_head, inv_temp, row_target, sb, store, m_blocks, n_blocks);
}
template <bool STATS>
static void launch_lmhead_any(const Shape& s, const int32_t* n_rows_dev, int M_max, const void* hf, const int32_t* x_rows,
                              const void* lm_head, float inv_temp, const int32_t* row_target, const SamplerBufs& sb,
                              float* store, hipStream_t st) {
  // Row tiling.  The vocabulary gives thousands of workgroups (many rounds per CU), so above 128 rows the
  // 96-row tile is used: it fits two workgroups per CU, and the statistics epilogue and the pipeline fill of
  // one overlap the matrix products of the other (measured at M = 576, V = 151936: 308 us against 372 us with
  // 192-row tiles, one workgroup per CU).
  const int mt = M_max <= 32 ? 1 : M_max <= 64 ? 2 : M_max <= 128 ? 4 : 3;
#define BS_LM(MT_) launch_lmhead_t<MT_, STATS>(s, n_rows_dev, M_max, hf, x_rows, lm_head, inv_temp, row_target, sb, store, st)
  switch (mt) {
    case 1: BS_LM(1); break;
    case 2: BS_LM(2); break;
    case 4: BS_LM(4); break;
    default: BS_LM(3);
  }
#undef BS_LM
}
void launch_lmhead_stats(const Shape& s, const Plan& p, int M_max, const void* hf, const void* lm_head, float inv_temp,
                         const SamplerBufs& sb, float* logits_debug, hipStream_t st) {
  launch_lmhead_any<true>(s, p.n_rows, M_max, hf, nullptr, lm_head, inv_temp, p.row_target, sb, logits_debug, st);
}
void launch_lmhead_rows(const Shape& s, int B, const void* hf, const void* lm_head, const SamplerBufs& sb,
                        hipStream_t st) {
  launch_lmhead_any<false>(s, nullptr, B, hf, sb.sel_row, lm_head, 1.0f, nullptr, sb, sb.sel_logits, st);
}
void launch_logit_stats(const Plan& p, int M_max, int V, const float* logits, float inv_temp, const SamplerBufs& sb,
                        hipStream_t st) {
  dim3 grid((V + kRowVtile - 1) / kRowVtile, M_max);
  hipLaunchKernelGGL(logit_stats_kernel, grid, dim3(256), 0, st, p, M_max, V, logits, inv_temp, sb);
}
void launch_q_stats(const Plan& p, int M_max, int V, const void* q_logits, int q_dtype, const SamplerBufs& sb,
                    hipStream_t st) {
  if (q_dtype == BS_F32) hipLaunchKernelGGL(q_stats_kernel<float>, dim3(M_max), dim3(256), 0, st, p, V, (const float*)q_logits, sb);
  else hipLaunchKernelGGL(q_stats_kernel<bf16>, dim3(M_max), dim3(256), 0, st, p, V, (const bf16*)q_logits, sb);
}
void launch_accept_scan(const Plan& p, int B, int k_max, int M_max, int n_vtiles, bool dense_q, float temperature,
                        int eos_id, int emit_bonus, const float* u_accept, const SamplerBufs& sb, const FilterArgs& filter,
                        int32_t* n_accepted, int32_t* out_tokens, int32_t* n_emitted, uint32_t* near_tie, hipStream_t st) {
  const float inv_temp = temperature > 0.f ? 1.0f / temperature : 1.0f;
  if (n_vtiles > 4 * kStatChunks) {
    hipLaunchKernelGGL(row_stats_fold_kernel, dim3((M_max + 31) / 32, kStatChunks), dim3(256), 0, st, p, M_max, n_vtiles, inv_temp, sb);
    hipLaunchKernelGGL(row_stats_kernel, dim3(M_max), dim3(256), 0, st, p, M_max, kStatChunks, inv_temp, sb, sb.fold_max,
                       sb.fold_sum, sb.fold_arg);
  } else {
    hipLaunchKernelGGL(row_stats_kernel, dim3(M_max), dim3(256), 0, st, p, M_max, n_vtiles, inv_temp, sb, sb.part_max,
                       sb.part_sum, sb.part_arg);
  }
  if (filter.on) launch_filter(p, M_max, temperature, filter, sb, st);      // needs row_max
  hipLaunchKernelGGL(accept_scan_kernel, dim3((B + 63) / 64), dim3(64), 0, st, p, B, k_max, dense_q ? 1 : 0, temperature,
                     eos_id, emit_bonus, filter.on, u_accept, sb, n_accepted, out_tokens, n_emitted, near_tie);
}
template <typename Q, bool FILT>
static void launch_sample_t(int B, int k_max, int V, const float* logit_base, bool rows_are_selected, const Q* q_logits,
                            float temperature, const float* u_sample, const SamplerBufs& sb, const int32_t* n_accepted,
                            int32_t* out_tokens, int32_t* n_emitted, uint32_t* near_tie, hipStream_t st) {
  const int sel = rows_are_selected ? 1 : 0;
  hipLaunchKernelGGL((sample_sum_kernel<Q, FILT>), dim3(kSampleChunks, B), dim3(256), 0, st, V, logit_base, sel, q_logits, temperature, sb);
  hipLaunchKernelGGL((sample_mass_kernel<Q, FILT>), dim3(kSampleChunks, B), dim3(256), 0, st, V, logit_base, sel, q_logits, temperature, sb);
  hipLaunchKernelGGL((sample_pick_kernel<Q, FILT>), dim3(B), dim3(kPickThreads), 0, st, V, logit_base, sel, q_logits, temperature, u_sample, sb,
                     n_accepted, k_max, out_tokens, n_emitted, near_tie);
}
void launch_sample(int B, int k_max, int V, const float* logit_base, bool rows_are_selected, const void* q_logits,
                   int q_dtype, float temperature, bool filter_on, const float* u_sample, const SamplerBufs& sb,
                   const int32_t* n_accepted, int32_t* out_tokens, int32_t* n_emitted, uint32_t* near_tie,
                   hipStream_t st) {
  if (temperature == 0.f) return;                    // the scan already emitted the arg-max tokens
  // the filtered kernels are instantiations of their own: the membership test costs the unfiltered path nothing
#define BS_SAMPLE(Q_, F_) launch_sample_t<Q_, F_>(B, k_max, V, logit_base, rows_are_selected, (const Q_*)q_logits, temperature, \
                                                  u_sample, sb, n_accepted, out_tokens, n_emitted, near_tie, st)
  if (q_logits && q_dtype == BS_BF16) { if (filter_on) BS_SAMPLE(bf16, true); else BS_SAMPLE(bf16, false); }
  else                                { if (filter_on) BS_SAMPLE(float, true); else BS_SAMPLE(float, false); }
#undef BS_SAMPLE
}
