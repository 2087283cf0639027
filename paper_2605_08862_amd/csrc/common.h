// Internal declarations shared by the translation units of libbubblespec (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/bubblespec.h"

typedef __bf16 bf16;
typedef _Float16 f16;

template <typename T> __device__ __forceinline__ float to_f32(T x);
template <> __device__ __forceinline__ float to_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f32<bf16>(bf16 x) { return (float)x; }
template <> __device__ __forceinline__ float to_f32<f16>(f16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ f16 from_f32<f16>(float x) { return (f16)x; }             // RNE
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return (bf16)x; }  // RNE

// ---------------------------------------------------------------------------------------------
// float16 range guard.  bf16 models keep every matrix operand that is produced during the step
// (normalised rows, rotated queries, appended K/V, attention output, gated MLP activation) in IEEE
// float16, whose largest finite value is 65504.  A producer converts four values at a time and
// tests the packed result: a float16 is infinite or NaN iff its exponent field is all ones, i.e.
// iff (bits & 0x7fff) + 0x0400 carries into bit 15.  When that happens (never for sane models) the
// values are saturated to +-65504 (NaN becomes 0) and BS_FAULT_RANGE is set in the status word, so
// that no infinity or NaN enters a matrix product silently.
// ---------------------------------------------------------------------------------------------
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ bool f16x4_out_of_range(f16x4 v) {
  const u32x2 u = __builtin_bit_cast(u32x2, v);
  return ((((u[0] & 0x7fff7fffu) + 0x04000400u) | ((u[1] & 0x7fff7fffu) + 0x04000400u)) & 0x80008000u) != 0u;
}
__device__ __forceinline__ float f16_saturate(float x) { return x != x ? 0.f : fminf(fmaxf(x, -65504.f), 65504.f); }
// (a, b, c, d) -> four float16 values, saturated and flagged if any leaves the float16 range
__device__ __forceinline__ f16x4 to_f16x4_guarded(float a, float b, float c, float d, int32_t* __restrict__ status) {
  f16x4 v = f16x4{(f16)a, (f16)b, (f16)c, (f16)d};
  if (f16x4_out_of_range(v)) {
    v = f16x4{(f16)f16_saturate(a), (f16)f16_saturate(b), (f16)f16_saturate(c), (f16)f16_saturate(d)};
    atomicOr(status, BS_FAULT_RANGE);
  }
  return v;
}

constexpr int kPage = BS_PAGE_TOKENS;   // tokens per KV page
constexpr int kTile = 32;               // tokens per MFMA tile inside a page (bf16 layout)

// ---------------------------------------------------------------------------------------------
// Element order inside one KV page (all heads of one layer, kPage tokens).
//
// float32 pages are row-major [head][token][d] for both K and V.
//
// Pages of bf16 models hold bf16-rounded values (the cache dtype) ENCODED as IEEE float16 (same 16
// bits per element; exact for 6.1e-5 <= |x| <= 65504), so that they are operands of the f16 MFMA
// with no conversion in the attention loop.  They are stored in the operand order of the 32x32x16
// MFMA so that the attention kernel's wave-wide 16-byte-per-lane loads are 1 KiB contiguous and
// feed the matrix unit with no LDS staging and no shuffles.  Per head a page is two tiles of 32 tokens.
//   K tile: S^T = K Q^T uses K as the A operand.  A-row m of the tile holds token
//           tau = 16*(m%8/4) + 4*(m/8) + m%4  (so that accumulator register i of lane group g
//           is token 16g+i), and lane (m, g) needs, at K-step s, d = g*D/2 + 8s + j (j = 0..7;
//           the contraction index may be permuted freely as long as Q uses the same order).
//   V tile: O^T = V^T P^T uses V^T as the A operand, 32 d-values per d-tile; lane (d%32, g) at
//           step t needs tokens 16g + 8t + j.
// ---------------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ size_t kv_page_elems(int Hkv, int D) { return (size_t)Hkv * kPage * D; }

__host__ __device__ __forceinline__ int k_index_f32(int D, int h, int tok, int d) { return (h * kPage + tok) * D + d; }
__host__ __device__ __forceinline__ int v_index_f32(int D, int h, int tok, int d) { return (h * kPage + tok) * D + d; }

__host__ __device__ __forceinline__ int k_tile_row(int tau) {   // token in tile -> A-row m
  return 4 * (tau / 16) + (tau % 4) + 8 * ((tau % 16) / 4);
}
__host__ __device__ __forceinline__ int k_index_bf16(int D, int h, int tok, int d) {
  int tile = tok / kTile, m = k_tile_row(tok % kTile);
  int g = d / (D / 2), r = d % (D / 2), s = r / 8, j = r % 8;
  return ((((h * 2 + tile) * (D / 16) + s) * 2 + g) * 32 + m) * 8 + j;
}
__host__ __device__ __forceinline__ int v_index_bf16(int D, int h, int tok, int d) {
  int tile = tok / kTile, tau = tok % kTile;
  int g = tau / 16, t = (tau % 16) / 8, j = tau % 8, dt = d / 32, dl = d % 32;
  return ((((((h * 2 + tile) * (D / 32) + dt) * 2 + t) * 2 + g) * 32 + dl) * 8) + j;
}
template <typename T> __host__ __device__ __forceinline__ int k_index(int D, int h, int tok, int d);
template <> __host__ __device__ __forceinline__ int k_index<float>(int D, int h, int tok, int d) { return k_index_f32(D, h, tok, d); }
template <> __host__ __device__ __forceinline__ int k_index<bf16>(int D, int h, int tok, int d) { return k_index_bf16(D, h, tok, d); }
template <> __host__ __device__ __forceinline__ int k_index<f16>(int D, int h, int tok, int d) { return k_index_bf16(D, h, tok, d); }
template <typename T> __host__ __device__ __forceinline__ int v_index(int D, int h, int tok, int d);
template <> __host__ __device__ __forceinline__ int v_index<f16>(int D, int h, int tok, int d) { return v_index_bf16(D, h, tok, d); }
template <> __host__ __device__ __forceinline__ int v_index<float>(int D, int h, int tok, int d) { return v_index_f32(D, h, tok, d); }
template <> __host__ __device__ __forceinline__ int v_index<bf16>(int D, int h, int tok, int d) { return v_index_bf16(D, h, tok, d); }

// ---------------------------------------------------------------------------------------------
// Device-side plan of one step (lives in the workspace; written by plan_kernel).
// ---------------------------------------------------------------------------------------------
struct Plan {
  int32_t* status;      // [1]   BS_FAULT_* bits (sticky until polled)
  int32_t* n_rows;      // [2]   M, T_d
  int32_t* row_start;   // [B+1] first packed row of sequence b (k_b+1 rows each)
  int32_t* draft_start; // [B+1] first packed draft row of sequence b (k_b rows each)
  int32_t* seq_k;       // [B]   validated k_b (-1: sequence skipped)
  int32_t* seq_c;       // [B]   committed length c_b
  int32_t* seq_slot;    // [B]   validated slot
  int32_t* row_seq;     // [M_max] sequence of packed row r
  int32_t* row_pos;     // [M_max] i in 0..k_b
  int32_t* row_tok;     // [M_max] input token of row r
  int32_t* row_target;  // [M_max] draft token judged by row r (-1: none)
  // attention work list (bf16 models): every sequence's token range is cut into chunks of chunk_tiles 32-token
  // tiles; the item at list position i is (sequence item_seq[i], chunk item_chunk[i]) and the list is ordered by
  // decreasing size (full chunks, then the shorter last chunks).  Sequence b has item_start[b+1] - item_start[b]
  // chunks; its chunk c owns SLOT item_start[b] + c, by which partial results are addressed
  int32_t* attn_meta;   // [2]   chunk_tiles, number of items
  int32_t* item_start;  // [B+1]
  int32_t* item_seq;    // [item capacity]
  int32_t* item_chunk;  // [item capacity]
  int32_t* attn_queue;  // [n_layers][8] next position of every XCD's work queue (zeroed by plan_kernel)
};

// Capacity of the attention work list for B sequences when the launch wants at least s_min (sequence, chunk)
// items (see plan_kernel): sum_b chunks(b) <= B + S with S <= 4 max(B, s_min).
__host__ __device__ __forceinline__ int attn_item_capacity(int B, int s_min) { return 5 * (B > s_min ? B : s_min); }
constexpr int kAttnMaxSmin = 256;

struct KvView {
  int n_pages, n_slots, max_pages;
  const int32_t* block_table;
  int32_t* ctx_len;
};

struct Shape {
  int L, d, Hq, Hkv, D, F, V, dtype;
  float eps, theta;
  int Nqkv() const { return (Hq + 2 * Hkv) * D; }
};

// ---- launchers (each .hip file defines its own kernels and these host wrappers) ---------------
// plan.hip
// attn_s_min > 0: also build the attention work list (wanted number of items, at most kAttnMaxSmin);
// attn_force_chunks > 0 (tests): chunk size such that the longest sequence has that many chunks.
void launch_plan(const Plan& p, const KvView& kv, int B, int k_max, int vocab, const int32_t* seq_slot,
                 const int32_t* last_token, const int32_t* draft_tokens, const int32_t* draft_len,
                 bool need_kv, int attn_s_min, int attn_force_chunks, int n_layers, hipStream_t st);
void launch_commit(const Plan& p, const KvView& kv, int B, const int32_t* seq_slot,
                   const int32_t* n_commit, hipStream_t st);
void launch_clear_status(int32_t* status, hipStream_t st);
void launch_kv_lengths(const KvView& kv, int B, const int32_t* seq_slot, int32_t* out, int32_t* status, hipStream_t st);
// elementwise.hip
// also fills the step's rotary tables cos_t / sin_t [M_max][D/2] (shared by all layers)
void launch_embed(const Shape& s, const Plan& p, int M_max, const void* embed, float* h, const double* inv_freq,
                  float* cos_t, float* sin_t, hipStream_t st);
// h[r] += sum of n_slabs slabs [M_max, d] (n_slabs may be 0), then out[r] = RMSNorm(h[r]).
struct SlabRule;
void launch_rmsnorm(const Shape& s, const Plan& p, int M_max, float* h, const float* slabs, const SlabRule& n_slabs,
                    const float* gain, void* out, hipStream_t st);
// qkv is the float32 projection, given as n_slabs >= 1 slabs [M_max, Nqkv] that are summed.
// inv_freq: [D/2] float64 table written by launch_rope_table.
void launch_rope_table(const Shape& s, double* inv_freq, hipStream_t st);
// cos_t / sin_t: [M_max][D/2] tables of the step's packed rows (filled by launch_embed, once per step).
void launch_rope_append(const Shape& s, const Plan& p, const KvView& kv, int M_max, const float* cos_t, const float* sin_t,
                        const float* qkv, int n_slabs, void* q_out, void* k_pages, void* v_pages, hipStream_t st);
void launch_kv_copy(const Shape& s, const KvView& kv, int slot, int pos0, int n, void* k_pages, void* v_pages,
                    void* k_rows, void* v_rows, bool to_pages, int32_t* status, hipStream_t st);
// qkv_rope.hip   QKV projection + rotary + KV append in one kernel (bf16 models with head size 128); A = normed
// rows (float16), Wp = packed wqkv.
bool qkv_rope_supported(const Shape& s);
void launch_qkv_rope(const Shape& s, const Plan& p, const KvView& kv, int M_max, const void* A, const void* Wp,
                     const float* cos_t, const float* sin_t, void* q_out, void* k_pages, void* v_pages, hipStream_t st);
// gemm.hip   C[M,N] (+)= A[M,K] * W[N,K]^T with an epilogue.  float32 models: A, W float32 row-major.
// bf16 models: A float16 row-major, W the packed float16 copy made by launch_pack_weight.
enum GemmEpilogue { EPI_STORE = 0, EPI_RESID_ADD = 1, EPI_SWIGLU = 2, EPI_STORE_F32 = 3 };
// Returns the number of K-split slabs written (bf16 models, EPI_RESID_ADD / EPI_STORE_F32: `out` is the
// slab buffer [split][M_max][N] and the consumer sums the slabs), or 0 when `out` was updated in place
// (float32 models).
constexpr int kMaxGemmSplit = 8;
// Number of K-split slabs a float32-epilogue GEMM writes: fixed on the host (bm == 0), or decided on the DEVICE from
// the step's row count M, which only the device knows (draft lengths may come straight from the lookup kernel): the
// launch is sized for the row limit, the kernel and the consumer of the slabs both evaluate slabs(M).  The rule: as
// many K splits (at most 4, at least 4 K tiles each) as keep all workgroups of the live row blocks resident at once.
__host__ __device__ __forceinline__ int gemm_adaptive_split(int tiles, int nk, int cap) {
  int s = tiles > 0 ? cap / tiles : 1;
  if (s > 4) s = 4;
  if (s > nk / 4) s = nk / 4;
  return s < 1 ? 1 : s;
}
struct SlabRule {
  int fixed;                    // slab count when bm == 0 (0: the output was updated in place)
  int bm, n_blocks, nk, cap;    // device rule: row tile, column blocks, K tiles, resident workgroups
  int bm_alt;                   // second row tile the producer may choose on the device (0: none)
  // Row tile of the step: with two candidates, the one whose launch is shorter by this model: all workgroups of a
  // round run at once, a workgroup's time ~ rows of its tile x K tiles of its split, and the 128-row loop does
  // about 5 % more work per unit of time.
  __host__ __device__ int tile_rows(int M) const {
    if (bm_alt == 0) return bm;
    long cost[2];
    for (int i = 0; i < 2; ++i) {
      const int b = i ? bm_alt : bm, tiles = ((M + b - 1) / b) * n_blocks, s = gemm_adaptive_split(tiles, nk, cap);
      const int rounds = (tiles * s + cap - 1) / cap;
      cost[i] = (long)b * ((nk + s - 1) / s) * (rounds > 0 ? rounds : 1) * (b == 128 ? 19 : 20);
    }
    return cost[1] < cost[0] ? bm_alt : bm;
  }
  __host__ __device__ int slabs(int M) const {
    if (bm == 0) return fixed;
    const int b = tile_rows(M);
    return gemm_adaptive_split(((M + b - 1) / b) * n_blocks, nk, cap);
  }
};
// status: the step's device status word (float16-range faults of the float16 epilogues).
SlabRule launch_gemm_resid(int dtype, const int32_t* n_rows_dev, int M_max, int N, int K, const void* A, const void* W,
                           void* out, int32_t* status, hipStream_t st);
int launch_gemm(int dtype, GemmEpilogue epi, const int32_t* n_rows_dev, int M_max, int N, int K,
                const void* A, const int32_t* a_rows /*optional gather*/, const void* W, void* out,
                int32_t* status, hipStream_t st);
size_t packed_weight_elems(int N, int K);
void launch_pack_weight(const void* w_bf16, int N, int K, void* packed_f16, int32_t* status, hipStream_t st);
// attention.hip
// attention_plan_params gives the work-list parameters launch_plan needs for the same (B, k_max);
// launch_attention_init clears the completion counters once, at context creation.
void attention_plan_params(const Shape& s, int B, int k_max, int* s_min, int* force_chunks);
void launch_attention_init(const Shape& s, int B_max, void* scratch, hipStream_t st);
void launch_attention(const Shape& s, const Plan& p, const KvView& kv, int layer, int B, int B_max, int k_max, int M_max,
                      const void* q, const void* k_pages, const void* v_pages, void* out, void* scratch,
                      void* prof_token, hipStream_t st);
void attention_prof_mark(void* token, hipStream_t st, bool begin);   // api.hip: event pair around the main kernel
size_t attention_scratch_bytes(const Shape& s, int B_max, int k_max);
// sampler.hip
struct SamplerBufs {
  float* part_max; float* part_sum; int32_t* part_arg;   // [n_vtiles, M_max]
  float* fold_max; float* fold_sum; int32_t* fold_arg;   // [16, M_max] tile entries folded over 16 vocabulary ranges
  float* z_target;                                       // [M_max] logit of the judged draft token
  float* row_max; float* row_lse; int32_t* row_arg;      // [M_max] combined statistics of each packed row
  float* q_max; float* q_lse; float* q_target;           // [M_max] per query row that judges a draft
  int32_t* sel_row; int32_t* sel_mode; int32_t* sel_qrow; int32_t* sel_tok; // [B_max]
  float* sel_pmax; float* sel_qmax;                      // [B_max] raw maxima of the sampled row / its q row
  double* samp_sum; double* samp_mass;                   // [B_max, 32 chunks, 2] sampling partials
  float* sel_logits;                                     // [B_max, V]
  uint32_t* f_key; int32_t* f_idx; float* f_lse;         // [M_max] top-k / top-p threshold of each row (filter.hip)
};

// Ranking key of a logit for the top-k / top-p filter: unsigned order == numeric order (-0 counts as +0), so
// "token j of row r is kept" reads  key > f_key[r] || (key == f_key[r] && j <= f_idx[r]).
__device__ __forceinline__ uint32_t filter_key(float z) {
  if (z == 0.0f) z = 0.0f;
  const uint32_t u = __float_as_uint(z);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ bool filter_keeps(uint32_t key, int j, uint32_t f_key, int f_idx) {
  return key > f_key || (key == f_key && j <= f_idx);
}
struct FilterArgs { int on; int top_k; float top_p; const float* logits; int V; };
int lmhead_vtiles(int V);
void launch_lmhead_stats(const Shape& s, const Plan& p, int M_max, const void* hf, const void* lm_head,
                         float inv_temp, const SamplerBufs& sb, float* logits_debug, hipStream_t st);
void launch_logit_stats(const Plan& p, int M_max, int V, const float* logits, float inv_temp,
                        const SamplerBufs& sb, hipStream_t st);
void launch_lmhead_rows(const Shape& s, int B, const void* hf, const void* lm_head, const SamplerBufs& sb,
                        hipStream_t st);
void launch_q_stats(const Plan& p, int M_max, int V, const void* q_logits, int q_dtype, const SamplerBufs& sb,
                    hipStream_t st);
void launch_accept_scan(const Plan& p, int B, int k_max, int M_max, int n_vtiles, bool dense_q, float temperature,
                        int eos_id, int emit_bonus, const float* u_accept, const SamplerBufs& sb, const FilterArgs& filter,
                        int32_t* n_accepted, int32_t* out_tokens, int32_t* n_emitted, uint32_t* near_tie, hipStream_t st);
void launch_sample(int B, int k_max, int V, const float* logit_base, bool rows_are_selected, const void* q_logits,
                   int q_dtype, float temperature, bool filter_on, const float* u_sample, const SamplerBufs& sb,
                   const int32_t* n_accepted, int32_t* out_tokens, int32_t* n_emitted, uint32_t* near_tie,
                   hipStream_t st);
// filter.hip   per-row threshold of the top-k / top-p filter (needs row_max of the same logits)
constexpr int kFilterMaxVocab = 262136;
void launch_filter(const Plan& p, int M_max, float temperature, const FilterArgs& filter, const SamplerBufs& sb,
                   hipStream_t st);
// index.hip   prebuilt suffix-automaton index: header check (host copy of the first 8 words) and the device walk
bool index_header_ok(const int32_t* header_host, size_t bytes, int* n_prompts);
void launch_index_lookup(const int32_t* blob, int n_prompts, const int32_t* seq_prompt, const int32_t* tail, int B,
                         int max_match, int min_match, int k_max, int32_t* draft_tokens, int32_t* draft_len,
                         hipStream_t st);
// lookup.hip
void launch_lookup(int B, int n_prompts, const int32_t* pool_tokens, const int64_t* rollout_offsets,
                   const int32_t* prompt_rollout_begin, const int32_t* seq_prompt, const int32_t* tail,
                   int max_match, int min_match, int k_max, int32_t* draft_tokens, int32_t* draft_len,
                   hipStream_t st);
