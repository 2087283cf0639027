// Prebuilt draft index (Sec. 3.2: the per-prompt suffix structure over pre-generated rollouts, with node
// occurrence counts; Alg. 1 "retrieve a draft block").
//
// bs_index_build (host) builds, per prompt, the suffix automaton of its rollouts joined by unique separators
// (so no match crosses a rollout boundary).  A state stands for a set of substrings with the same set of end
// positions; the size of that set is the number of occurrences of those substrings.  The retrieval rule
// ("longest suffix of the last tokens that occurs in the pool, then repeatedly the token that follows the most
// occurrences, ties to the smaller id") becomes: walk the context from the root, then follow a precomputed
// `best` edge per state, i.e. O(m + k) dependent loads per sequence instead of a scan of the prompt's pool.
// The blob is position independent (int32 arrays); the caller copies it to the device and binds it.
//
//   header[8]: magic, n_prompts, n_states, n_edges, 0...
//   prompt_root[n_prompts]         first state (root) of each prompt's automaton, -1 for an empty pool
//   edge_begin[n_states + 1]       edges of state v: edge_begin[v] .. edge_begin[v+1], sorted by token
//   best_tok[n_states], best_next[n_states]   most frequent successor token (-1: none) and its state
//   edge_tok[n_edges], edge_next[n_edges]
#include "common.h"
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

namespace {
constexpr int32_t kIndexMagic = 0x42535849;   // "BSXI"

struct Automaton {
  std::vector<int32_t> len, link, cnt, head;            // per state; head = first edge of the state's list
  std::vector<int64_t> e_tok;                           // per edge (separators are negative 64-bit values)
  std::vector<int32_t> e_next, e_chain;                 // target state, next edge of the same state
  std::vector<int32_t> table;                           // open addressing: edge index + 1, 0 = empty
  size_t mask = 0;

  static uint64_t mix(uint64_t x) { x ^= x >> 33; x *= 0xff51afd7ed558ccdull; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ull; return x ^ (x >> 33); }
  size_t slot_of(int32_t st, int64_t tok) const { return (size_t)mix(((uint64_t)(uint32_t)st << 40) ^ (uint64_t)tok) & mask; }

  void reserve(size_t n_tokens) {
    size_t cap = 64;
    while (cap < 8 * (n_tokens + 2)) cap <<= 1;         // <= 3n edges (+ copies for clones): load factor < 1/2
    table.assign(cap, 0);
    mask = cap - 1;
    len.reserve(2 * n_tokens + 2); link.reserve(2 * n_tokens + 2); cnt.reserve(2 * n_tokens + 2); head.reserve(2 * n_tokens + 2);
  }
  int32_t new_state(int32_t l) { len.push_back(l); link.push_back(-1); cnt.push_back(0); head.push_back(-1); return (int32_t)len.size() - 1; }
  int32_t find_edge(int32_t st, int64_t tok) const {
    for (size_t s = slot_of(st, tok);; s = (s + 1) & mask) {
      const int32_t e = table[s];
      if (e == 0) return -1;
      if (e_tok[e - 1] == tok && e_src[e - 1] == st) return e - 1;
    }
  }
  std::vector<int32_t> e_src;
  void set_edge(int32_t st, int64_t tok, int32_t to) {
    const int32_t e = find_edge(st, tok);
    if (e >= 0) { e_next[e] = to; return; }
    e_tok.push_back(tok); e_next.push_back(to); e_src.push_back(st); e_chain.push_back(head[st]);
    head[st] = (int32_t)e_tok.size() - 1;
    size_t s = slot_of(st, tok);
    while (table[s] != 0) s = (s + 1) & mask;
    table[s] = (int32_t)e_tok.size();
  }
  int32_t last = 0;
  void extend(int64_t c) {
    const int32_t cur = new_state(len[last] + 1);
    cnt[cur] = 1;
    int32_t p = last;
    while (p != -1 && find_edge(p, c) < 0) { set_edge(p, c, cur); p = link[p]; }
    if (p == -1) {
      link[cur] = 0;
    } else {
      const int32_t q = e_next[find_edge(p, c)];
      if (len[p] + 1 == len[q]) {
        link[cur] = q;
      } else {
        const int32_t clone = new_state(len[p] + 1);
        for (int32_t e = head[q]; e >= 0; e = e_chain[e]) set_edge(clone, e_tok[e], e_next[e]);
        link[clone] = link[q];
        while (p != -1) {
          const int32_t e = find_edge(p, c);
          if (e < 0 || e_next[e] != q) break;
          e_next[e] = clone;
          p = link[p];
        }
        link[q] = clone;
        link[cur] = clone;
      }
    }
    last = cur;
  }
  // occurrence counts: every non-clone state ends at one position; a state's end positions include those of
  // the states that link to it
  void count() {
    const int32_t n = (int32_t)len.size();
    int32_t max_len = 0;
    for (int32_t v = 0; v < n; ++v) max_len = std::max(max_len, len[v]);
    std::vector<int32_t> bucket(max_len + 2, 0), order(n);
    for (int32_t v = 0; v < n; ++v) ++bucket[len[v] + 1];
    for (int32_t l = 0; l <= max_len; ++l) bucket[l + 1] += bucket[l];
    for (int32_t v = 0; v < n; ++v) order[bucket[len[v]]++] = v;
    for (int32_t i = n - 1; i > 0; --i) { const int32_t v = order[i]; if (link[v] >= 0) cnt[link[v]] += cnt[v]; }
  }
};

// Eight lanes per sequence: lane i tries the suffix of length mm - i of the context (all candidate lengths at once
// instead of one after the other: the walk is a chain of dependent loads, and the root's edge list alone is a
// 17-step binary search for a 150k-token vocabulary); the longest that occurs wins and lane 0 follows the
// precomputed best edges.
__global__ void __launch_bounds__(64) index_lookup_kernel(const int32_t* __restrict__ blob, int n_prompts_ctx,
                                                          const int32_t* __restrict__ seq_prompt,
                                                          const int32_t* __restrict__ tail, int B, int max_match,
                                                          int min_match, int k_max, int32_t* __restrict__ draft_tokens,
                                                          int32_t* __restrict__ draft_len) {
  const int sub = threadIdx.x & 7;
  const int b = blockIdx.x * 8 + (threadIdx.x >> 3);
  const bool live = b < B;
  const int bb = live ? b : B - 1;                       // idle lanes shadow the last sequence (no stores)
  const int n_prompts = blob[1], n_states = blob[2], n_edges = blob[3];
  const int32_t* prompt_root = blob + 8;
  const int32_t* edge_begin = prompt_root + n_prompts;
  const int32_t* best_tok = edge_begin + n_states + 1;
  const int32_t* best_next = best_tok + n_states;
  const int32_t* edge_tok = best_next + n_states;
  const int32_t* edge_next = edge_tok + n_edges;
  const int pr = seq_prompt[bb];
  const bool usable = pr >= 0 && pr < n_prompts && pr < n_prompts_ctx && k_max > 0 && prompt_root[pr] >= 0 &&
                      prompt_root[pr] < n_states;
  const int32_t* ctx = tail + (size_t)bb * max_match;
  int mm = 0;                                            // usable context: trailing non-padding entries
  while (mm < max_match && ctx[max_match - 1 - mm] >= 0) ++mm;
  const int m = mm - sub;                                // this lane's candidate length (max_match <= 8)
  int st = -1;
  if (usable && m >= min_match) {
    int v = prompt_root[pr];
    for (int i = 0; i < m && v >= 0; ++i) {
      const int tok = ctx[max_match - m + i];
      int lo = min(max(edge_begin[v], 0), n_edges), hi = min(max(edge_begin[v + 1], lo), n_edges);
      int found = -1;
      while (lo < hi) {                                  // edges of a state are sorted by token
        const int mid = (lo + hi) >> 1, t = edge_tok[mid];
        if (t == tok) { found = edge_next[mid]; break; }
        if (t < tok) lo = mid + 1; else hi = mid;
      }
      v = (found >= 0 && found < n_states) ? found : -1;
    }
    st = v;
  }
  int chosen = -1;                                       // longest candidate that occurs = smallest lane index
  const int base = threadIdx.x & ~7;
#pragma unroll
  for (int i = 7; i >= 0; --i) {
    const int s_i = __shfl(st, base + i);
    if (s_i >= 0) chosen = s_i;
  }
  if (!live || sub != 0) return;
  int32_t* out = draft_tokens + (size_t)b * k_max;
  int n_draft = 0;
  st = chosen;
  while (st >= 0 && n_draft < k_max) {                   // most frequent continuation, state by state
    const int t = best_tok[st];
    if (t < 0) break;
    out[n_draft++] = t;
    const int nx = best_next[st];
    st = (nx >= 0 && nx < n_states) ? nx : -1;
  }
  for (int i = n_draft; i < k_max; ++i) out[i] = -1;
  draft_len[b] = n_draft;
}
}  // namespace

void launch_index_lookup(const int32_t* blob, int n_prompts, const int32_t* seq_prompt, const int32_t* tail, int B,
                         int max_match, int min_match, int k_max, int32_t* draft_tokens, int32_t* draft_len,
                         hipStream_t st) {
  hipLaunchKernelGGL(index_lookup_kernel, dim3((B + 7) / 8), dim3(64), 0, st, blob, n_prompts, seq_prompt, tail, B,
                     max_match, min_match, k_max, draft_tokens, draft_len);
}

bool index_header_ok(const int32_t* header_host, size_t bytes, int* n_prompts) {
  if (!header_host || bytes < 8 * sizeof(int32_t) || header_host[0] != kIndexMagic) return false;
  const long long np = header_host[1], ns = header_host[2], ne = header_host[3];
  if (np < 1 || ns < 0 || ne < 0) return false;
  if ((size_t)(8 + np + (ns + 1) + 2 * ns + 2 * ne) * sizeof(int32_t) != bytes) return false;
  *n_prompts = (int)np;
  return true;
}

extern "C" {

bs_status bs_index_build(int n_prompts, const int32_t* pool_tokens, const int64_t* rollout_offsets,
                         const int32_t* prompt_rollout_begin, void** blob_out, size_t* bytes_out) {
  if (!blob_out || !bytes_out) return BS_EINVAL;
  *blob_out = nullptr;
  *bytes_out = 0;
  if (n_prompts < 1 || !pool_tokens || !rollout_offsets || !prompt_rollout_begin) return BS_EINVAL;
  try {
    std::vector<int32_t> prompt_root(n_prompts, -1), edge_begin(1, 0), best_tok, best_next, edge_tok, edge_next;
    for (int pr = 0; pr < n_prompts; ++pr) {
      const int r0 = prompt_rollout_begin[pr], r1 = prompt_rollout_begin[pr + 1];
      if (r0 < 0 || r1 < r0) return BS_EINVAL;
      const int64_t t0 = rollout_offsets[r0], t1 = rollout_offsets[r1];
      if (t0 < 0 || t1 < t0) return BS_EINVAL;
      if (t1 == t0) continue;                            // no tokens: no automaton
      if ((t1 - t0) + (r1 - r0) > (int64_t)0x1fffffff) return BS_ESHAPE;
      Automaton a;
      a.reserve((size_t)(t1 - t0) + (size_t)(r1 - r0));
      a.new_state(0);
      for (int r = r0; r < r1; ++r) {
        const int64_t s0 = rollout_offsets[r], s1 = rollout_offsets[r + 1];
        if (s1 < s0 || s0 < t0 || s1 > t1) return BS_EINVAL;     // offsets must be non-decreasing
        for (int64_t i = s0; i < s1; ++i) {
          if (pool_tokens[i] < 0) return BS_EINVAL;
          a.extend(pool_tokens[i]);
        }
        a.extend(-1 - (int64_t)(r - r0));                // unique separator: nothing matches across it
      }
      a.count();
      const int32_t base = (int32_t)best_tok.size(), n = (int32_t)a.len.size();
      if ((int64_t)base + n > (int64_t)0x7ffffff0) return BS_ESHAPE;
      prompt_root[pr] = base;
      std::vector<std::pair<int32_t, int32_t>> edges;
      for (int32_t v = 0; v < n; ++v) {
        edges.clear();
        for (int32_t e = a.head[v]; e >= 0; e = a.e_chain[e])
          if (a.e_tok[e] >= 0) edges.emplace_back((int32_t)a.e_tok[e], a.e_next[e]);
        std::sort(edges.begin(), edges.end());
        int32_t bt = -1, bn = -1, bc = 0;
        for (const auto& e : edges) {
          edge_tok.push_back(e.first);
          edge_next.push_back(base + e.second);
          if (a.cnt[e.second] > bc) { bc = a.cnt[e.second]; bt = e.first; bn = base + e.second; }   // sorted: ties keep the smaller id
        }
        best_tok.push_back(bt);
        best_next.push_back(bn);
        if (edge_tok.size() > (size_t)0x7ffffff0) return BS_ESHAPE;
        edge_begin.push_back((int32_t)edge_tok.size());
      }
    }
    const size_t ns = best_tok.size(), ne = edge_tok.size();
    const size_t words = 8 + (size_t)n_prompts + (ns + 1) + 2 * ns + 2 * ne;
    int32_t* blob = new (std::nothrow) int32_t[words];
    if (!blob) return BS_ECAPACITY;
    int32_t* w = blob;
    const int32_t header[8] = {kIndexMagic, n_prompts, (int32_t)ns, (int32_t)ne, 0, 0, 0, 0};
    std::memcpy(w, header, sizeof(header)); w += 8;
    std::memcpy(w, prompt_root.data(), n_prompts * sizeof(int32_t)); w += n_prompts;
    std::memcpy(w, edge_begin.data(), (ns + 1) * sizeof(int32_t)); w += ns + 1;
    std::memcpy(w, best_tok.data(), ns * sizeof(int32_t)); w += ns;
    std::memcpy(w, best_next.data(), ns * sizeof(int32_t)); w += ns;
    std::memcpy(w, edge_tok.data(), ne * sizeof(int32_t)); w += ne;
    std::memcpy(w, edge_next.data(), ne * sizeof(int32_t));
    *blob_out = blob;
    *bytes_out = words * sizeof(int32_t);
    return BS_OK;
  } catch (const std::bad_alloc&) {
    return BS_ECAPACITY;
  }
}

void bs_index_free(void* blob) { delete[] (int32_t*)blob; }

}  // extern "C"
