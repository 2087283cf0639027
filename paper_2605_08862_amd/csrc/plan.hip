// Device-side planning of one verify step, KV commit, status word.
//
// draft_len may be produced on the device by the lookup kernel, so the packing of the ragged
// query rows (Alg. 1: every sequence verifies its own block of k_b drafts; Sec. 3.3: all query
// lengths ride in one batch) is computed here, on the device, with no host round trip.
#include "common.h"

__global__ void __launch_bounds__(256) plan_kernel(Plan p, KvView kv, int B, int k_max, int vocab,
                                                   const int32_t* __restrict__ seq_slot,
                                                   const int32_t* __restrict__ last_token,
                                                   const int32_t* __restrict__ draft_tokens,
                                                   const int32_t* __restrict__ draft_len, int need_kv, int attn_s_min,
                                                   int attn_force_chunks, int n_layers) {
  __shared__ int s_fault;
  __shared__ int s_slot[4096];                      // B <= 4096 (checked at context creation)
  __shared__ int s_k[4096];                         // validated k_b (-1: skipped)
  __shared__ int s_c[4096];                         // c_b
  __shared__ int s_pr[256], s_pt[256];              // per-thread partial row / draft counts, then their prefix
  const int tid = threadIdx.x;
  if (tid == 0) s_fault = 0;
  if (need_kv)
    for (int b = tid; b < B; b += blockDim.x) s_slot[b] = seq_slot[b];
  __syncthreads();
  // phase 1: per-sequence validation.  Four lanes share a sequence: each repeats the scalar checks (same addresses:
  // one transaction) and takes a quarter of the duplicate-slot scan and of the block-table entries, eight loads at a
  // time, so that a context of 2048 tokens (33 pages) costs two memory round trips instead of five.
  for (int b = tid >> 2; b < B; b += blockDim.x >> 2) {
    const int sub = tid & 3;
    int k = draft_len[b], fault = 0, c = 0, slot = 0;
    if (k < 0 || k > k_max) { fault |= BS_FAULT_DRAFT_LEN; }
    if (need_kv) {
      slot = s_slot[b];
      if (slot < 0 || slot >= kv.n_slots) {
        fault |= BS_FAULT_SLOT;
      } else {
        for (int b2 = sub; b2 < b; b2 += 4) if (s_slot[b2] == slot) fault |= BS_FAULT_SLOT;
        c = kv.ctx_len[slot];
        if (!(fault & BS_FAULT_DRAFT_LEN)) {
          if (c < 0 || (long)c + k + 1 > (long)kv.max_pages * kPage) {
            fault |= BS_FAULT_KV_PAGES;
          } else {
            const int32_t* bt = kv.block_table + (size_t)slot * kv.max_pages;
            const int last = (c + k) / kPage;
            for (int pg0 = sub * 8; pg0 <= last; pg0 += 32) {
              int id[8];
#pragma unroll
              for (int u = 0; u < 8; ++u) id[u] = bt[min(pg0 + u, last)];
#pragma unroll
              for (int u = 0; u < 8; ++u) if (id[u] < 0 || id[u] >= kv.n_pages) fault |= BS_FAULT_KV_PAGES;
            }
          }
        }
      }
    }
    // token ids of the sequence's rows (the last token and the k drafts), a quarter per lane: a sequence with an id
    // outside the vocabulary is skipped like one with a bad draft length (no row is embedded, appended or judged)
    if (!(fault & BS_FAULT_DRAFT_LEN)) {
      if (sub == 0 && last_token) {
        const int t = last_token[b];
        if (t < 0 || t >= vocab) fault |= BS_FAULT_TOKEN_ID;
      }
      for (int i = sub; i < k; i += 4) {
        const int t = draft_tokens[(size_t)b * k_max + i];
        if (t < 0 || t >= vocab) fault |= BS_FAULT_TOKEN_ID;
      }
    }
    fault |= __shfl_xor(fault, 1);
    fault |= __shfl_xor(fault, 2);
    if (sub == 0) {
      p.seq_k[b] = fault ? -1 : k;
      s_k[b] = fault ? -1 : k;
      s_c[b] = c;
      p.seq_c[b] = c;
      p.seq_slot[b] = slot;
      if (fault) atomicOr(&s_fault, fault);
    }
  }
  __syncthreads();
  // phase 2: prefix sums over the sequences (each thread a contiguous range, partials scanned by thread 0)
  const int per = (B + 255) / 256;
  const int b_lo = min(tid * per, B), b_hi = min(b_lo + per, B);
  {
    int r = 0, t = 0;
    for (int b = b_lo; b < b_hi; ++b) if (s_k[b] >= 0) { r += s_k[b] + 1; t += s_k[b]; }
    s_pr[tid] = r; s_pt[tid] = t;
  }
  __syncthreads();
  if (tid == 0) {
    int r = 0, t = 0;
    for (int i = 0; i < 256; ++i) { const int a = s_pr[i], c2 = s_pt[i]; s_pr[i] = r; s_pt[i] = t; r += a; t += c2; }
    p.row_start[B] = r;
    p.draft_start[B] = t;
    p.n_rows[0] = r;
    p.n_rows[1] = t;
  }
  __syncthreads();
  {
    int r = s_pr[tid], t = s_pt[tid];
    for (int b = b_lo; b < b_hi; ++b) {
      p.row_start[b] = r;
      p.draft_start[b] = t;
      if (s_k[b] >= 0) { r += s_k[b] + 1; t += s_k[b]; }
    }
  }
  __syncthreads();
  // phase 3: per-row maps (parallel over sequences x positions)
  for (int idx = tid; idx < B * (k_max + 1); idx += blockDim.x) {
    int b = idx / (k_max + 1), i = idx % (k_max + 1);
    int k = s_k[b];
    if (k < 0 || i > k) continue;
    int r = p.row_start[b] + i;
    // every id was validated in phase 1 (a sequence with a bad one has s_k[b] = -1 and is skipped above)
    const int tok = (i == 0) ? (last_token ? last_token[b] : 0) : draft_tokens[(size_t)b * k_max + i - 1];
    const int tgt = (i < k) ? draft_tokens[(size_t)b * k_max + i] : -1;
    p.row_seq[r] = b;
    p.row_pos[r] = i;
    p.row_tok[r] = tok;
    p.row_target[r] = tgt;
  }
  __syncthreads();
  if (tid == 0 && s_fault) atomicOr(p.status, s_fault);
  if (!need_kv || attn_s_min <= 0) return;
  for (int i = tid; i < 8 * n_layers; i += blockDim.x) p.attn_queue[i] = 0;

  // phase 4: attention work list.  The (sequence, KV head) streams of a ragged batch differ in length by
  // orders of magnitude (contexts of 512 .. 32768 tokens in one step), so the token range of every sequence
  // is cut into chunks of a common size; the attention kernel's persistent workgroups walk the (sequence,
  // chunk) items.  T = tiles in total, S0 = max(B, s_min) = items that fill the GPU once:
  //   * lengths within 25 % of their mean: chunk = ceil(1.25 T / S0) if S0 = B (one chunk per sequence: no
  //     partial results), ceil(T / S0) if the batch is smaller than s_min (equal chunks, one round);
  //   * ragged batch: chunk = ceil(T / s_min), one workgroup's fair share of the step: a longer sequence is cut
  //     into fair shares, the shorter ones and the last chunks are whole items, and the list hands them out in
  //     decreasing size (see the ordering below), so the queues run dry on the smallest items.  Measured on the
  //     long-tail batch (128 sequences of 512 .. 32768 tokens, 7B heads): chunks of 1/4, 1/2, 3/4, 1, 1.5 and 2 fair
  //     shares take 335, 310, 301, 297, 393 and 483 us per layer.
  // sum_b chunks(b) <= B + T / chunk <= B + 4 S0 always (the work list's capacity).
  __shared__ int s_red[256];
  __shared__ int s_cht;
  auto tiles_of = [&](int b) { return s_k[b] < 0 ? 0 : (s_c[b] + s_k[b] + 1 + kTile - 1) / kTile; };
  {
    int t = 0, mx = 0, nv = 0;
    for (int b = b_lo; b < b_hi; ++b) { const int n = tiles_of(b); t += n; mx = max(mx, n); nv += n > 0; }
    s_pr[tid] = t; s_red[tid] = mx; s_pt[tid] = nv;
  }
  __syncthreads();
  if (tid == 0) {
    long long T = 0; int mx = 0; long long s_valid = 0;
    for (int i = 0; i < 256; ++i) { T += s_pr[i]; mx = max(mx, s_red[i]); s_valid += s_pt[i]; }
    const int S = max(B, attn_s_min), cap = attn_item_capacity(B, attn_s_min);
    long long cht = (S > B) ? (T + S - 1) / S : (5 * T + 4LL * S - 1) / (4LL * S);
    if (4LL * mx * s_valid > 5 * T) cht = (T + attn_s_min - 1) / attn_s_min;   // ragged: longest > 1.25 x mean
    if (attn_force_chunks > 0) cht = (mx + attn_force_chunks - 1) / attn_force_chunks;
    const long long floor_cht = (T + (cap - B) - 1) / (cap - B);      // keeps sum_b ceil(n_b / cht) <= cap
    if (cht < floor_cht) cht = floor_cht;
    if (cht < 1) cht = 1;
    s_cht = (int)min(cht, (long long)0x3fffffff);
  }
  __syncthreads();
  const int cht = s_cht;
  // Order of the list = order in which the persistent workgroups take the items: every chunk of full size first,
  // then the last (shorter) chunk of every sequence, longest first (64 size classes), so that the work still
  // handed out when the queues run dry is the smallest there is.  item_start[b] keeps numbering a sequence's
  // chunks contiguously (slot item_start[b] + chunk): the partial results are addressed by slot, not by position.
  __shared__ int s_hist[64], s_base[64];
  auto chunks_of = [&](int b) { return (tiles_of(b) + cht - 1) / cht; };
  auto size_class = [&](int rem) { return 63 - min(63, (int)(((long long)rem * 64 - 1) / cht)); };   // rem in 1 .. cht
  {
    int n = 0, nf = 0;
    for (int b = b_lo; b < b_hi; ++b) { const int nc = chunks_of(b); n += nc; nf += max(nc - 1, 0); }
    s_pr[tid] = n; s_pt[tid] = nf;
  }
  if (tid < 64) s_hist[tid] = 0;
  __syncthreads();
  if (tid == 0) {
    int n = 0, nf = 0;
    for (int i = 0; i < 256; ++i) { const int a = s_pr[i], f = s_pt[i]; s_pr[i] = n; s_pt[i] = nf; n += a; nf += f; }
    p.item_start[B] = n;
    p.attn_meta[0] = cht;
    p.attn_meta[1] = n;
    s_red[0] = nf;                                       // full-size chunks that are not the last of their sequence
  }
  __syncthreads();
  {
    int n = s_pr[tid], pf = s_pt[tid];
    for (int b = b_lo; b < b_hi; ++b) {
      p.item_start[b] = n;
      const int nc = chunks_of(b);
      for (int c = 0; c + 1 < nc; ++c, ++pf) { p.item_seq[pf] = b; p.item_chunk[pf] = c; }
      if (nc > 0) atomicAdd(&s_hist[size_class(tiles_of(b) - (nc - 1) * cht)], 1);
      n += nc;
    }
  }
  __syncthreads();
  if (tid == 0) {
    int at = s_red[0];
    for (int i = 0; i < 64; ++i) { s_base[i] = at; at += s_hist[i]; s_hist[i] = 0; }
  }
  __syncthreads();
  for (int b = b_lo; b < b_hi; ++b) {
    const int nc = chunks_of(b);
    if (nc == 0) continue;
    const int cl = size_class(tiles_of(b) - (nc - 1) * cht);
    const int pos = s_base[cl] + atomicAdd(&s_hist[cl], 1);
    p.item_seq[pos] = b;
    p.item_chunk[pos] = nc - 1;
  }
}

__global__ void commit_kernel(Plan p, KvView kv, int B, const int32_t* __restrict__ seq_slot,
                              const int32_t* __restrict__ n_commit) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int k = p.seq_k[b];
  if (k < 0) return;                       // sequence was skipped by the verify step
  int n = n_commit[b];
  if (n < 0 || n > k + 1 || seq_slot[b] != p.seq_slot[b]) { atomicOr(p.status, BS_FAULT_COMMIT); return; }
  kv.ctx_len[p.seq_slot[b]] = p.seq_c[b] + n;
}

__global__ void clear_status_kernel(int32_t* status) { *status = 0; }

// out[b] = committed length of slot seq_slot[b] (-1 and BS_FAULT_SLOT for a slot outside the cache)
__global__ void kv_lengths_kernel(KvView kv, int B, const int32_t* __restrict__ seq_slot, int32_t* __restrict__ out,
                                  int32_t* __restrict__ status) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int slot = seq_slot[b];
  if (slot < 0 || slot >= kv.n_slots) { out[b] = -1; atomicOr(status, BS_FAULT_SLOT); return; }
  out[b] = kv.ctx_len[slot];
}

void launch_plan(const Plan& p, const KvView& kv, int B, int k_max, int vocab, const int32_t* seq_slot,
                 const int32_t* last_token, const int32_t* draft_tokens, const int32_t* draft_len,
                 bool need_kv, int attn_s_min, int attn_force_chunks, int n_layers, hipStream_t st) {
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(256), 0, st, p, kv, B, k_max, vocab, seq_slot, last_token,
                     draft_tokens, draft_len, need_kv ? 1 : 0, attn_s_min, attn_force_chunks, n_layers);
}
void launch_commit(const Plan& p, const KvView& kv, int B, const int32_t* seq_slot, const int32_t* n_commit,
                   hipStream_t st) {
  hipLaunchKernelGGL(commit_kernel, dim3((B + 255) / 256), dim3(256), 0, st, p, kv, B, seq_slot, n_commit);
}
void launch_kv_lengths(const KvView& kv, int B, const int32_t* seq_slot, int32_t* out, int32_t* status, hipStream_t st) {
  hipLaunchKernelGGL(kv_lengths_kernel, dim3((B + 255) / 256), dim3(256), 0, st, kv, B, seq_slot, out, status);
}
void launch_clear_status(int32_t* status, hipStream_t st) {
  hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(1), 0, st, status);
}
