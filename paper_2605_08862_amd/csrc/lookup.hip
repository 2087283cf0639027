// Draft retrieval (Sec. 3.2, Alg. 1 "retrieve a draft block"): for every sequence, find the
// longest suffix of its rollout (up to max_match tokens) that occurs in its prompt's pool of
// pre-generated rollouts and walk the most frequent continuation for up to k_max tokens.
//
// The paper builds a suffix tree on the CPU and walks it per query.  On MI355X a prompt's whole
// pool (tens of thousands of tokens, a few hundred KB) streams through one workgroup in a few
// microseconds, so this kernel scans the raw pool (one workgroup per sequence) and keeps the
// surviving occurrences in LDS; it returns exactly what a counted suffix-trie walk returns.
// Occurrence counting uses an LDS hash table; when more distinct successors exist than the
// table holds, the vocabulary is split into residue classes and counted class by class, so the
// result is exact for any pool.
#include "common.h"

namespace {
constexpr int kCap = 1024;     // occurrences kept in LDS; beyond that the pool is rescanned per step
constexpr int kHash = 4096;    // hash slots (token, count)
constexpr int kMaxMatch = 8;
constexpr int kThreads = 1024;  // one workgroup per sequence: many loads in flight hide the pool's latency

struct Best { int cnt; int tok; };
__device__ __forceinline__ bool better(int c1, int t1, int c2, int t2) { return c1 > c2 || (c1 == c2 && t1 < t2); }
}  // namespace

__global__ void __launch_bounds__(kThreads) lookup_kernel(int n_prompts, const int32_t* __restrict__ pool,
                                                     const int64_t* __restrict__ ro, const int32_t* __restrict__ prb,
                                                     const int32_t* __restrict__ seq_prompt,
                                                     const int32_t* __restrict__ tail, int max_match, int min_match,
                                                     int k_max, int32_t* __restrict__ draft_tokens,
                                                     int32_t* __restrict__ draft_len) {
  __shared__ int s_cnt[kMaxMatch + 1];
  __shared__ int s_pos[2][kCap], s_end[2][kCap];   // offsets from the prompt's first pool token
  __shared__ int s_ncand[2];
  __shared__ int s_htok[kHash], s_hcnt[kHash];
  __shared__ int s_flag, s_best_cnt, s_best_tok;
  __shared__ int s_ctx[kMaxMatch];
  __shared__ int s_draft[BS_MAX_K + 1];
  const int b = blockIdx.x, tid = threadIdx.x;
  int32_t* out = draft_tokens + (size_t)b * k_max;
  for (int i = tid; i < k_max; i += kThreads) out[i] = -1;
  const int pr = seq_prompt[b];
  if (pr < 0 || pr >= n_prompts || k_max == 0) { if (tid == 0) draft_len[b] = 0; return; }
  const int r_begin = prb[pr], r_end = prb[pr + 1];
  const long long base = ro[r_begin];
  if (tid < max_match) s_ctx[tid] = tail[(size_t)b * max_match + tid];
  if (tid <= kMaxMatch) s_cnt[tid] = 0;
  __syncthreads();
  int mm = 0;                                       // usable context length: trailing non-padding entries
  while (mm < max_match && s_ctx[max_match - 1 - mm] >= 0) ++mm;

  // match length of the context ending at pool position e inside rollout [s0, s1)
  auto match_len = [&](long long e, long long s0) {
    int len = 0;
    while (len < mm && e - len >= s0 && pool[e - len] == s_ctx[max_match - 1 - len]) ++len;
    return len;
  };
  // phase 1 (one pass over the pool): histogram of match lengths; every occurrence of at least
  // min_match tokens is also kept (with its length) while the list has room, so that the usual case
  // needs no second pass
  if (tid == 0) { s_ncand[0] = 0; s_ncand[1] = 0; }
  __syncthreads();
  // kScan positions per thread and iteration: their tokens are requested together and only positions whose
  // token equals the newest context token go on to the full comparison (one dependent load per position
  // and iteration left the scan bound by memory latency)
  constexpr int kScan = 8;
  const int newest = mm > 0 ? s_ctx[max_match - 1] : -2;     // pool tokens are >= 0
  for (int r = r_begin; r < r_end; ++r) {
    const long long s0 = ro[r], s1 = ro[r + 1];
    for (long long e0 = s0 + tid; e0 < s1; e0 += (long long)kThreads * kScan) {
      int tok[kScan];
#pragma unroll
      for (int u = 0; u < kScan; ++u) {
        const long long e = e0 + (long long)u * kThreads;
        tok[u] = e < s1 ? pool[e] : -1;
      }
#pragma unroll
      for (int u = 0; u < kScan; ++u) {
        if (tok[u] != newest) continue;
        const long long e = e0 + (long long)u * kThreads;
        int len = match_len(e, s0);
        if (len >= min_match) {
          atomicAdd(&s_cnt[len], 1);
          int i = atomicAdd(&s_ncand[1], 1);           // total count (may exceed the capacity)
          if (i < kCap) { s_pos[1][i] = (int)(e - base); s_end[1][i] = (int)(s1 - base); s_htok[i] = len; }
        }
      }
    }
  }
  __syncthreads();
  int m_star = 0, n0 = 0;
  for (int m = mm; m >= min_match; --m) {
    n0 += s_cnt[m];
    if (n0 > 0) { m_star = m; break; }
  }
  if (m_star == 0) { if (tid == 0) draft_len[b] = 0; return; }
  const bool list_mode = n0 <= kCap;
  const int n_all = s_ncand[1];
  __syncthreads();
  if (list_mode) {
    if (n_all <= kCap) {                                // filter the kept occurrences by the chosen length
      for (int i = tid; i < n_all; i += kThreads)
        if (s_htok[i] >= m_star) {
          int o = atomicAdd(&s_ncand[0], 1);
          s_pos[0][o] = s_pos[1][i];
          s_end[0][o] = s_end[1][i];
        }
    } else {                                            // the kept list overflowed: second pass for m_star only
      for (int r = r_begin; r < r_end; ++r) {
        const long long s0 = ro[r], s1 = ro[r + 1];
        for (long long e = s0 + tid; e < s1; e += kThreads)
          if (match_len(e, s0) >= m_star) {
            int i = atomicAdd(&s_ncand[0], 1);
            s_pos[0][i] = (int)(e - base);
            s_end[0][i] = (int)(s1 - base);
          }
      }
    }
    __syncthreads();
  }

  int n_draft = 0, cur = 0;
  for (int j = 0; j < k_max; ++j) {
    // enumerate the successor token of every surviving occurrence
    auto for_each_succ = [&](auto f) {
      if (list_mode) {
        for (int i = tid; i < s_ncand[cur]; i += kThreads) {
          int e = s_pos[cur][i];
          if (e + 1 < s_end[cur][i]) f(pool[base + e + 1]);
        }
      } else {
        for (int r = r_begin; r < r_end; ++r) {
          const long long s0 = ro[r], s1 = ro[r + 1];
          for (long long e = s0 + tid; e + j + 1 < s1; e += kThreads) {
            if (match_len(e, s0) < m_star) continue;
            bool ok = true;
            for (int i = 0; i < j && ok; ++i) ok = pool[e + 1 + i] == s_draft[i];
            if (ok) f(pool[e + j + 1]);
          }
        }
      }
    };
    // most frequent successor (ties: smaller id), counted class by class if the table overflows
    int best_cnt = 0, best_tok = 0x7fffffff;
    for (int P = 1;; P *= 2) {
      bool overflow = false;
      best_cnt = 0; best_tok = 0x7fffffff;
      for (int cls = 0; cls < P; ++cls) {
        for (int i = tid; i < kHash; i += kThreads) { s_htok[i] = -1; s_hcnt[i] = 0; }
        if (tid == 0) { s_flag = 0; s_best_cnt = 0; s_best_tok = 0x7fffffff; }
        __syncthreads();
        for_each_succ([&](int t) {
          if (P > 1 && (t & (P - 1)) != cls) return;
          unsigned h = ((unsigned)t * 2654435761u) >> 20;          // 12 bits
          for (int probe = 0; probe < kHash; ++probe) {
            int slot = (h + probe) & (kHash - 1);
            int old = atomicCAS(&s_htok[slot], -1, t);
            if (old == -1 || old == t) { atomicAdd(&s_hcnt[slot], 1); return; }
          }
          s_flag = 1;
        });
        __syncthreads();
        if (s_flag) { overflow = true; }
        // reduce the table (each thread its slots, then one atomic round through LDS)
        int c = 0, t = 0x7fffffff;
        for (int i = tid; i < kHash; i += kThreads)
          if (s_htok[i] >= 0 && better(s_hcnt[i], s_htok[i], c, t)) { c = s_hcnt[i]; t = s_htok[i]; }
        if (c > 0) atomicMax(&s_best_cnt, c);
        __syncthreads();
        if (c > 0 && c == s_best_cnt) atomicMin(&s_best_tok, t);
        __syncthreads();
        if (better(s_best_cnt, s_best_tok, best_cnt, best_tok)) { best_cnt = s_best_cnt; best_tok = s_best_tok; }
        __syncthreads();
        if (overflow) break;
      }
      if (!overflow) break;
    }
    if (best_cnt == 0) break;
    if (tid == 0) { s_draft[j] = best_tok; out[j] = best_tok; }
    ++n_draft;
    if (list_mode) {
      const int nxt = cur ^ 1;
      if (tid == 0) s_ncand[nxt] = 0;
      __syncthreads();
      for (int i = tid; i < s_ncand[cur]; i += kThreads) {
        int e = s_pos[cur][i];
        if (e + 1 < s_end[cur][i] && pool[base + e + 1] == best_tok) {
          int o = atomicAdd(&s_ncand[nxt], 1);
          s_pos[nxt][o] = e + 1;
          s_end[nxt][o] = s_end[cur][i];
        }
      }
      cur = nxt;
    }
    __syncthreads();
  }
  if (tid == 0) draft_len[b] = n_draft;
}

void launch_lookup(int B, int n_prompts, const int32_t* pool_tokens, const int64_t* rollout_offsets,
                   const int32_t* prompt_rollout_begin, const int32_t* seq_prompt, const int32_t* tail, int max_match,
                   int min_match, int k_max, int32_t* draft_tokens, int32_t* draft_len, hipStream_t st) {
  hipLaunchKernelGGL(lookup_kernel, dim3(B), dim3(kThreads), 0, st, n_prompts, pool_tokens, rollout_offsets,
                     prompt_rollout_begin, seq_prompt, tail, max_match, min_match, k_max, draft_tokens, draft_len);
}
