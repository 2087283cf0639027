// Top-k / top-p filtering of the target distribution: Sec. 3.2 defines p_t as the decoding distribution "after
// temperature scaling and any top-p / top-k filtering".  Reading taken: tokens are ranked by logit (equal logits:
// lower index first); top-k keeps the first k of the ranking; top-p then keeps the shortest prefix of what is left
// whose mass reaches top_p times the mass of what is left; the kept probabilities are renormalised.
//
// The kept set of a row is always a prefix of the ranking, so it is described by a threshold: the ranking key of
// its last token and, among tokens with exactly that logit, the largest index kept.  One workgroup per row finds
// it by radix descent over the 32-bit ranking key (11 + 11 + 10 bits), reading the float32 logits of the row
// once per level:
//   top-k   histogram of COUNTS of the keys that match the prefix found so far; the bin that holds the k-th
//           largest key extends the prefix;
//   top-p   the same with histograms of MASS, exp(z/T - max) in float64 turned into 45-bit fixed point so that
//           the 64-bit integer sums do not depend on the order of the atomic additions: the result is the same
//           on every run, and a row's total is exact to 2^-46 per token.  The bin in which the running mass
//           (from the top) reaches the target extends the prefix.
// Tokens whose logit equals the threshold have equal mass; how many of them are needed follows by division, and
// which (the lowest indices) by a counting pass that runs only when not all of them are kept.
// The mass of the kept set (for the renormalisation in the accept test) comes out of the same integers.
//
// Reading a 600 KB row once per level (up to eight times) would be the whole cost, so after the first level of a
// descent the tokens of the one bin that holds the threshold are copied to a list in LDS (as 39-bit composites: the
// 21 key bits below the bin, then the inverted index, so that no two are equal and ties need no special case) and
// the remaining levels walk that list.  The first pass of the mass descent doubles as the list-building pass of
// top-k, so a row is read two or three times.  Where a bin holds more tokens than the list (a constant row,
// heavily quantised logits, the nucleus boundary of a flat row) the descent goes on from the level it has reached
// with one pass over the row per level.
#include "common.h"
#include <limits.h>

namespace {
typedef unsigned long long u64;
typedef float f4 __attribute__((ext_vector_type(4)));
constexpr double kScale = 35184372088832.0;                  // 2^45: V < 2^18 tokens of mass <= 1 stay below 2^63
constexpr int kLevels = 3;
__device__ __constant__ const int kBits[kLevels] = {11, 11, 10};

constexpr int kCand = 2048;                                  // candidate list entries (LDS); three workgroups fit a CU
constexpr int kIdxBits = 18, kLowBits = 21, kCompBits = kIdxBits + kLowBits;
constexpr u64 kIdxMask = (1ull << kIdxBits) - 1;

struct Shared {
  uint32_t hist_c[2048];
  u64 hist_m[2048];
  u64 hist_l[1024];                                          // levels over the candidate list
  u64 scan[256];
  u64 above;
  int bin;
  int cand_n;
  u64 cand[kCand];
};

// composite of a token inside its first-level bin: larger = earlier in the ranking
__device__ __forceinline__ u64 composite(uint32_t key, int j) {
  return ((u64)(key & ((1u << kLowBits) - 1)) << kIdxBits) | (kIdxMask - (u64)j);
}

// f(j, z_j) for every token of the row; eight 16-byte loads in flight per thread (a workgroup per row is limited by
// the bytes it keeps in flight, not by HBM)
template <typename F>
__device__ __forceinline__ void for_each_logit(const float* __restrict__ z, int V, F f) {
  const int tid = threadIdx.x;
  const int nvec = (((uintptr_t)z) & 15) == 0 ? V / 4 : 0;
  int i = tid;
  for (; i + 7 * 256 < nvec; i += 8 * 256) {
    f4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = *(const f4*)(z + 4 * (size_t)(i + u * 256));
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) f(4 * (i + u * 256) + e, v[u][e]);
  }
  for (; i < nvec; i += 256) {
    const f4 a = *(const f4*)(z + 4 * (size_t)i);
#pragma unroll
    for (int e = 0; e < 4; ++e) f(4 * i + e, a[e]);
  }
  for (int j = nvec * 4 + tid; j < V; j += 256) f(j, z[j]);
}

// Walks the nb bins from the highest down: the first bin at which the running sum reaches `target` (>= 1) goes to
// sh.bin and the sum of the bins above it to sh.above; sh.bin = -1 if the total stays below the target.
// All 256 threads call it; the histogram must be complete (barrier before).
template <typename T>
__device__ void find_crossing(const T* hist, int nb, u64 target, Shared& sh) {
  const int tid = threadIdx.x, per = nb / 256;
  u64 s = 0;
  for (int i = 0; i < per; ++i) s += hist[nb - 1 - (tid * per + i)];
  sh.scan[tid] = s;
  if (tid == 0) sh.bin = -1;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const u64 v = tid >= o ? sh.scan[tid - o] : 0;
    __syncthreads();
    sh.scan[tid] += v;
    __syncthreads();
  }
  const u64 incl = sh.scan[tid], excl = incl - s;
  if (excl < target && incl >= target) {
    u64 acc = excl;
    for (int i = 0; i < per; ++i) {
      const int bin = nb - 1 - (tid * per + i);
      const u64 h = hist[bin];
      if (acc + h >= target) { sh.bin = bin; sh.above = acc; break; }
      acc += h;
    }
  }
  __syncthreads();
}

// Index of the n-th (1-based) token in index order that satisfies pred; V - 1 if there are fewer.  Each thread
// takes one contiguous slice.  Runs only for rows whose threshold logit is shared by more tokens than are kept.
template <typename P>
__device__ int nth_match(const float* __restrict__ z, int V, int n, P pred, Shared& sh) {
  const int tid = threadIdx.x, slice = (V + 255) / 256;
  const int j0 = min(tid * slice, V), j1 = min(j0 + slice, V);
  int cnt = 0;
  for (int j = j0; j < j1; ++j) cnt += pred(j, z[j]) ? 1 : 0;
  __syncthreads();
  sh.scan[tid] = (u64)cnt;
  if (tid == 0) sh.bin = V - 1;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const u64 v = tid >= o ? sh.scan[tid - o] : 0;
    __syncthreads();
    sh.scan[tid] += v;
    __syncthreads();
  }
  const int incl = (int)sh.scan[tid], excl = incl - cnt;
  if (excl < n && incl >= n) {
    int seen = excl;
    for (int j = j0; j < j1; ++j)
      if (pred(j, z[j]) && ++seen == n) { sh.bin = j; break; }
  }
  __syncthreads();
  const int r = sh.bin;
  __syncthreads();
  return r;
}

// Walks the composites of the candidate list from the largest down, adding weight(c) (1 when counting, the token's
// mass otherwise) of the candidates with c >= floor_c: returns the composite at which the running sum reaches
// `target` (>= 1, <= the total) and puts the sum of the weights before it into sh.above.  Composites are unique,
// so the four levels (10 + 10 + 10 + 9 bits) end at exactly one candidate.
template <typename Wt>
__device__ u64 list_select(Shared& sh, int n, u64 floor_c, u64 target, Wt weight) {
  const int tid = threadIdx.x;
  u64 prefix = 0, before = 0;
  int done = 0;
  for (int lvl = 0; lvl < 4; ++lvl) {
    const int bits = lvl < 3 ? 10 : 9, nb = 1 << bits, shift = kCompBits - done - bits;
    for (int i = tid; i < nb; i += 256) sh.hist_l[i] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += 256) {
      const u64 c = sh.cand[i];
      if (c >= floor_c && (done == 0 || (c >> (kCompBits - done)) == prefix))
        atomicAdd(&sh.hist_l[(c >> shift) & (u64)(nb - 1)], weight(c));
    }
    __syncthreads();
    find_crossing(sh.hist_l, nb, target, sh);
    const int bin = max(sh.bin, 0);
    target -= sh.above;
    before += sh.above;
    prefix = (prefix << bits) | (u64)bin;
    done += bits;
    __syncthreads();
  }
  if (tid == 0) sh.above = before;
  __syncthreads();
  return prefix;
}

__global__ void __launch_bounds__(256) filter_kernel(Plan p, int M_max, int V, const float* __restrict__ logits,
                                                     float temperature, int top_k, float top_p, SamplerBufs sb) {
  extern __shared__ __align__(16) char lds_raw[];
  Shared& sh = *(Shared*)lds_raw;
  const int m = blockIdx.x, tid = threadIdx.x;
  if (m >= min(p.n_rows[0], M_max)) return;
  const float* z = logits + (size_t)m * V;
  const double inv_T = 1.0 / (double)temperature;
  const double mxp = (double)sb.row_max[m] * inv_T;
  const bool use_k = top_k > 0 && top_k < V, use_p = top_p < 1.0f;
  auto mass = [&](float zj) -> u64 { return (u64)(exp((double)zj * inv_T - mxp) * kScale + 0.5); };
  auto value_of = [](uint32_t key) { return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key); };

  // State of the two descents.  The short way below fills it in; where a bin is too large for the candidate list
  // it leaves the descent at the level it reached and the long way (one row pass per level) continues from there.
  uint32_t kk = 0;                                           // top-k threshold: ranking key and index cut
  int cut_k = INT_MAX;
  bool k_known = !use_k;
  uint32_t k_prefix = 0, k_need = (uint32_t)top_k;           // top-k descent: key bits found, tokens still to take
  int k_done = 0, k_lvl = 0;
  uint32_t prefix = 0;                                       // mass descent: key bits found, mass still to reach
  int done = 0, m_lvl = 0, cut = INT_MAX;
  u64 target = 0, kept_mass = 0;
  bool finished = false;

  // ================= short way: first level from the row, the rest from a candidate list in LDS
  {
    bool ok = true;
    int b1 = -1;                                             // first-level bin of the top-k threshold (-1: no top-k)
    if (use_k) {
      for (int i = tid; i < 2048; i += 256) sh.hist_c[i] = 0;
      __syncthreads();
      for_each_logit(z, V, [&](int, float zj) { atomicAdd(&sh.hist_c[filter_key(zj) >> kLowBits], 1u); });
      __syncthreads();
      find_crossing(sh.hist_c, 2048, (u64)top_k, sh);
      b1 = max(sh.bin, 0);
      k_need = (uint32_t)top_k - (uint32_t)sh.above;
      k_prefix = (uint32_t)b1;
      k_done = kBits[0];
      k_lvl = 1;
      ok = sh.hist_c[b1] <= (uint32_t)kCand;
      __syncthreads();
    }
    if (ok) {
      // pass over the row: masses of the tokens that are certainly in the top-k set, counts per bin, and the list
      // of the tokens of bin b1
      for (int i = tid; i < 2048; i += 256) { sh.hist_m[i] = 0; sh.hist_c[i] = 0; }
      if (tid == 0) sh.cand_n = 0;
      __syncthreads();
      for_each_logit(z, V, [&](int j, float zj) {
        const uint32_t key = filter_key(zj);
        const int l1 = (int)(key >> kLowBits);
        if (l1 > b1) {
          atomicAdd(&sh.hist_m[l1], mass(zj));
          atomicAdd(&sh.hist_c[l1], 1u);
        } else if (l1 == b1) {
          const int slot = atomicAdd(&sh.cand_n, 1);
          if (slot < kCand) sh.cand[slot] = composite(key, j);
        }
      });
      __syncthreads();
      u64 c_k = 0;                                           // composite of the last token of the top-k set
      int n_list = 0;
      if (use_k) {
        n_list = min(sh.cand_n, kCand);
        c_k = list_select(sh, n_list, 0, (u64)k_need, [](u64) -> u64 { return 1; });
        const uint32_t hi = (uint32_t)b1 << kLowBits;
        kk = hi | (uint32_t)(c_k >> kIdxBits);
        cut_k = (int)(kIdxMask - (c_k & kIdxMask));
        k_known = true;
        for (int i = tid; i < n_list; i += 256) {
          const u64 c = sh.cand[i];
          if (c >= c_k) atomicAdd(&sh.hist_m[b1], mass(value_of(hi | (uint32_t)(c >> kIdxBits))));
        }
        __syncthreads();
      }
      u64 part = 0;
      for (int i = tid; i < 2048; i += 256) part += sh.hist_m[i];
      if (tid == 0) sh.above = 0;
      __syncthreads();
      atomicAdd(&sh.above, part);
      __syncthreads();
      const u64 total = sh.above;
      __syncthreads();
      if (!use_p) {
        prefix = kk; cut = cut_k; kept_mass = total; finished = true;
      } else {
        const double td = (double)top_p * (double)total;
        target = (u64)td;
        if ((double)target < td) ++target;
        if (target < 1) target = 1;
        if (target > total) target = total;
        find_crossing(sh.hist_m, 2048, target, sh);
        const int bf = max(sh.bin, 0);                       // first-level bin of the final threshold
        target -= sh.above;
        kept_mass = sh.above;
        prefix = (uint32_t)bf;
        done = kBits[0];
        m_lvl = 1;
        __syncthreads();
        if (bf != b1) {                                      // another bin: its tokens are all in the top-k set
          ok = sh.hist_c[bf] <= (uint32_t)kCand;
          __syncthreads();
          if (ok) {
            if (tid == 0) sh.cand_n = 0;
            __syncthreads();
            for_each_logit(z, V, [&](int j, float zj) {
              const uint32_t key = filter_key(zj);
              if ((int)(key >> kLowBits) == bf) {
                const int slot = atomicAdd(&sh.cand_n, 1);
                if (slot < kCand) sh.cand[slot] = composite(key, j);
              }
            });
            __syncthreads();
            n_list = min(sh.cand_n, kCand);
            c_k = 0;
          }
        }
        if (ok) {
          const uint32_t hi = (uint32_t)bf << kLowBits;
          const u64 c_f = list_select(sh, n_list, c_k, target, [&](u64 c) -> u64 { return mass(value_of(hi | (uint32_t)(c >> kIdxBits))); });
          prefix = hi | (uint32_t)(c_f >> kIdxBits);
          cut = (int)(kIdxMask - (c_f & kIdxMask));
          kept_mass += sh.above + mass(value_of(prefix));
          finished = true;
          __syncthreads();
        }
      }
    }
    __syncthreads();
  }

  // ================= long way: every remaining level reads the row
  if (!k_known) {
    uint32_t eq = 0;
    for (int lvl = k_lvl; lvl < kLevels; ++lvl) {
      const int bits = kBits[lvl], nb = 1 << bits, shift = 32 - k_done - bits;
      for (int i = tid; i < nb; i += 256) sh.hist_c[i] = 0;
      __syncthreads();
      for_each_logit(z, V, [&](int, float zj) {
        const uint32_t key = filter_key(zj);
        if (k_done == 0 || (key >> (32 - k_done)) == k_prefix) atomicAdd(&sh.hist_c[(key >> shift) & (nb - 1)], 1u);
      });
      __syncthreads();
      find_crossing(sh.hist_c, nb, k_need, sh);
      const int bin = max(sh.bin, 0);                      // a crossing always exists: k_need <= tokens under the prefix
      k_need -= (uint32_t)sh.above;
      k_prefix = (k_prefix << bits) | (uint32_t)bin;
      eq = sh.hist_c[bin];
      k_done += bits;
      __syncthreads();
    }
    kk = k_prefix;
    if (eq > k_need) cut_k = nth_match(z, V, (int)k_need, [&](int, float zj) { return filter_key(zj) == kk; }, sh);
  }
  auto in_topk = [&](uint32_t key, int j) { return !use_k || filter_keeps(key, j, kk, cut_k); };

  // ---- mass of the top-k set and, with top-p, the shortest prefix of it that reaches top_p of that mass
  for (int lvl = m_lvl; lvl < kLevels && !finished; ++lvl) {
    const int bits = kBits[lvl], nb = 1 << bits, shift = 32 - done - bits;
    for (int i = tid; i < nb; i += 256) sh.hist_m[i] = 0;
    __syncthreads();
    for_each_logit(z, V, [&](int j, float zj) {
      const uint32_t key = filter_key(zj);
      if ((done == 0 || (key >> (32 - done)) == prefix) && in_topk(key, j))
        atomicAdd(&sh.hist_m[(key >> shift) & (nb - 1)], mass(zj));
    });
    __syncthreads();
    if (lvl == 0) {
      // total mass of the top-k set (integer additions: any order gives the same sum)
      u64 part = 0;
      for (int i = tid; i < nb; i += 256) part += sh.hist_m[i];
      if (tid == 0) sh.above = 0;
      __syncthreads();
      atomicAdd(&sh.above, part);
      __syncthreads();
      const u64 total = sh.above;
      __syncthreads();
      if (!use_p) { kept_mass = total; prefix = kk; cut = cut_k; finished = true; continue; }
      const double td = (double)top_p * (double)total;
      target = (u64)td;
      if ((double)target < td) ++target;
      if (target < 1) target = 1;
      if (target > total) target = total;
    }
    find_crossing(sh.hist_m, nb, target, sh);
    const int bin = max(sh.bin, 0);                        // a crossing always exists: 1 <= target <= mass under the prefix
    target -= sh.above;
    kept_mass += sh.above;
    prefix = (prefix << bits) | (uint32_t)bin;
    done += bits;
    if (lvl == kLevels - 1) {
      // all tokens of this bin have the same logit, hence the same mass q_e: ceil(target / q_e) of them are kept
      const u64 bin_mass = sh.hist_m[bin];
      u64 q_e = mass(value_of(prefix));
      if (q_e == 0) q_e = 1;                               // not reached: the bin holds mass
      const u64 n_eq = bin_mass / q_e, n_need = (target + q_e - 1) / q_e;
      kept_mass += n_need * q_e;
      __syncthreads();
      if (n_need < n_eq) {
        const uint32_t kp = prefix;
        cut = nth_match(z, V, (int)n_need, [&](int j, float zj) { const uint32_t key = filter_key(zj); return key == kp && in_topk(key, j); }, sh);
      } else {
        cut = (use_k && prefix == kk) ? cut_k : INT_MAX;
      }
    }
    __syncthreads();
  }
  if (tid == 0) {
    sb.f_key[m] = prefix;
    sb.f_idx[m] = cut;
    sb.f_lse[m] = (float)(mxp + log((double)kept_mass / kScale));
  }
}
}  // namespace

void launch_filter(const Plan& p, int M_max, float temperature, const FilterArgs& f, const SamplerBufs& sb, hipStream_t st) {
  static bool attr_set = false;                              // more than 64 KiB of dynamic LDS needs an opt-in
  if (!attr_set) { (void)hipFuncSetAttribute((const void*)filter_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Shared)); attr_set = true; }
  hipLaunchKernelGGL(filter_kernel, dim3(M_max), dim3(256), sizeof(Shared), st, p, M_max, f.V, f.logits, temperature, f.top_k, f.top_p, sb);
}
