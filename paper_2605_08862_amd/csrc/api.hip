// C ABI of libbubblespec: argument validation, workspace carving and kernel sequencing of one
// speculative-verification step (Alg. 1 of the paper; see include/bubblespec.h for the contract).
#include "common.h"
#include <mutex>
#include <new>
#include <string>
#include <vector>

struct bs_ctx {
  Shape s;
  KvView kv;
  int B_max, k_max, M_max;
  std::vector<const float*> attn_norm, mlp_norm;
  std::vector<const void*> wqkv, wo, w_gate_up, w_down;   // GEMM operands: raw (float32) or packed float16 copies
  std::vector<void*> k_pages, v_pages;
  const void *embed, *lm_head;
  const float* final_norm;
  // workspace
  Plan plan;
  float* h;            // residual stream  [M_max, d] float32
  double* inv_freq;    // [D/2] rotary frequencies
  float *rope_cos, *rope_sin;   // [M_max, D/2] cos / sin of the step's rotary angles
  std::vector<void*> pk_qkv, pk_o, pk_gu, pk_down;         // bf16 models: packed copies in the workspace
  void* pk_lm = nullptr;
  void* a;             // normed rows      [M_max, d] (GEMM operand type: float32 / float16)
  float* qkv;          // [M_max, (Hq+2Hkv) D] float32 projection (rounded once, after the rotation)
  void* q;             // [M_max, Hq D] rotated queries
  float* slabs;        // bf16 models: K-split slabs of the float32 GEMM epilogues [8][M_max, max(Nqkv, d)]
  void* attn_out;      // [M_max, Hq D]
  void* act;           // [M_max, F]
  void* hf;            // final-norm rows  [M_max, d]
  void* attn_scratch;
  float* full_logits;  // float32 models only: [M_max, V]
  SamplerBufs sb;
  int n_vtiles;
  // pool
  int n_prompts = 0, n_rollouts = 0;
  const int32_t* pool_tokens = nullptr;
  const int64_t* rollout_offsets = nullptr;
  const int32_t* prompt_rollout_begin = nullptr;
  // measurement hooks
  const int32_t* index_blob = nullptr;   // device copy of a bs_index_build blob (optional)
  int index_prompts = 0;
  int prof_class = 0;
  int top_k = 0;              // top-k / top-p filter of the target distribution (bs_set_filter); 0 / 1.0 = off
  float top_p = 1.0f;
  float* filter_logits = nullptr;   // bf16 models: caller's [M_max, V] float32 scratch for the filtered path
  bool unfused_qkv = false;   // test hook: QKV GEMM + separate rotary kernel instead of the fused kernel
  std::vector<hipEvent_t> prof_ev;     // pairs (start, stop), created on first use
  size_t prof_used = 0;
  hipEvent_t prof_pending_stop = nullptr;
  // state
  bool verify_pending = false;
  int last_B = 0, last_k_max = 0;
  std::string err;
};

namespace {

struct Carver {
  char* base;
  size_t off = 0;
  template <typename T> T* take(size_t n) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? (T*)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

size_t elt(int dtype) { return dtype == BS_F32 ? 4 : 2; }

bs_status check_desc(const bs_model_desc* d, int B_max, int k_max) {
  if (!d) return BS_EINVAL;
  if (d->dtype != BS_F32 && d->dtype != BS_BF16) return BS_EINVAL;
  if (d->d_model > 16384) return BS_ESHAPE;               // the normalisation kernel keeps a row in registers
  if (d->n_layers < 1 || d->d_model < 64 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->d_ffn < 64 || d->vocab < 2)
    return BS_ESHAPE;
  if (d->head_dim != 64 && d->head_dim != 128) return BS_ESHAPE;
  if (d->d_model % 64 || d->d_ffn % 64 || d->n_q_heads % d->n_kv_heads) return BS_ESHAPE;
  if (B_max < 1 || B_max > 4096 || k_max < 0 || k_max > BS_MAX_K) return BS_ESHAPE;
  if (!(d->rms_eps >= 0.f) || !(d->rope_theta > 0.f)) return BS_EINVAL;
  // bf16 attention packs the (k_max+1)*G query rows of one KV head into at most four 32-row MFMA tiles
  if (d->dtype == BS_BF16 && (k_max + 1) * (d->n_q_heads / d->n_kv_heads) > 128) return BS_ESHAPE;
  return BS_OK;
}

// Plan arrays of B sequences / M packed rows; with_attention also lays out the attention work list.
void carve_plan(Carver& w, Plan& p, int B, int M, bool with_attention, int n_layers) {
  p.status = w.take<int32_t>(64);
  p.n_rows = w.take<int32_t>(64);
  p.row_start = w.take<int32_t>(B + 1);
  p.draft_start = w.take<int32_t>(B + 1);
  p.seq_k = w.take<int32_t>(B);
  p.seq_c = w.take<int32_t>(B);
  p.seq_slot = w.take<int32_t>(B);
  p.row_seq = w.take<int32_t>(M);
  p.row_pos = w.take<int32_t>(M);
  p.row_tok = w.take<int32_t>(M);
  p.row_target = w.take<int32_t>(M);
  if (!with_attention) {
    p.attn_meta = p.item_start = p.item_seq = p.item_chunk = p.attn_queue = nullptr;
    return;
  }
  p.attn_meta = w.take<int32_t>(64);
  p.item_start = w.take<int32_t>(B + 1);
  p.item_seq = w.take<int32_t>(attn_item_capacity(B, kAttnMaxSmin));
  p.item_chunk = w.take<int32_t>(attn_item_capacity(B, kAttnMaxSmin));
  p.attn_queue = w.take<int32_t>((size_t)8 * n_layers);
}

// Sampler buffers of B sequences / M packed rows with n_vtiles statistics tiles per row (sel_logits and the
// filter thresholds are laid out by the caller that needs them).
void carve_sampler(Carver& w, SamplerBufs& sb, int B, int M, int n_vtiles) {
  sb.part_max = w.take<float>((size_t)n_vtiles * M);
  sb.part_sum = w.take<float>((size_t)n_vtiles * M);
  sb.part_arg = w.take<int32_t>((size_t)n_vtiles * M);
  sb.fold_max = w.take<float>((size_t)16 * M);
  sb.fold_sum = w.take<float>((size_t)16 * M);
  sb.fold_arg = w.take<int32_t>((size_t)16 * M);
  sb.z_target = w.take<float>(M);
  sb.row_max = w.take<float>(M);
  sb.row_lse = w.take<float>(M);
  sb.row_arg = w.take<int32_t>(M);
  sb.q_max = w.take<float>(M);
  sb.q_lse = w.take<float>(M);
  sb.q_target = w.take<float>(M);
  sb.sel_pmax = w.take<float>(B);
  sb.sel_qmax = w.take<float>(B);
  sb.samp_sum = w.take<double>((size_t)B * 32 * 2);
  sb.samp_mass = w.take<double>((size_t)B * 32 * 2);
  sb.sel_row = w.take<int32_t>(B);
  sb.sel_mode = w.take<int32_t>(B);
  sb.sel_qrow = w.take<int32_t>(B);
  sb.sel_tok = w.take<int32_t>(B);
  sb.f_key = w.take<uint32_t>(M);
  sb.f_idx = w.take<int32_t>(M);
  sb.f_lse = w.take<float>(M);
  sb.sel_logits = nullptr;
}

// Lays the workspace out; with base == nullptr only measures it.
size_t carve(bs_ctx* c, char* base) {
  Carver w{base};
  const Shape& s = c->s;
  const int B = c->B_max, M = c->M_max;
  carve_plan(w, c->plan, B, M, true, s.L);
  c->h = w.take<float>((size_t)M * s.d);
  c->inv_freq = w.take<double>(64);
  c->rope_cos = w.take<float>((size_t)M * 64);
  c->rope_sin = w.take<float>((size_t)M * 64);
  c->a = w.take<char>((size_t)M * s.d * elt(s.dtype));          // float16 and bf16 have the same size
  c->qkv = w.take<float>((size_t)M * s.Nqkv());
  c->q = w.take<char>((size_t)M * s.Hq * s.D * elt(s.dtype));
  c->slabs = (s.dtype == BS_BF16)
                 ? w.take<float>((size_t)kMaxGemmSplit * M * (s.Nqkv() > s.d ? s.Nqkv() : s.d))
                 : nullptr;
  c->attn_out = w.take<char>((size_t)M * s.Hq * s.D * elt(s.dtype));
  c->act = w.take<char>((size_t)M * s.F * elt(s.dtype));
  c->hf = w.take<char>((size_t)M * s.d * elt(s.dtype));
  c->attn_scratch = w.take<char>(attention_scratch_bytes(s, B, c->k_max));
  c->n_vtiles = lmhead_vtiles(s.V);
  SamplerBufs& sb = c->sb;
  carve_sampler(w, sb, B, M, c->n_vtiles);
  if (s.dtype == BS_F32) {
    c->full_logits = w.take<float>((size_t)M * s.V);
    sb.sel_logits = nullptr;
  } else {
    c->full_logits = nullptr;
    sb.sel_logits = w.take<float>((size_t)B * s.V);
    c->pk_qkv.assign(s.L, nullptr); c->pk_o.assign(s.L, nullptr); c->pk_gu.assign(s.L, nullptr); c->pk_down.assign(s.L, nullptr);
    for (int l = 0; l < s.L; ++l) {
      c->pk_qkv[l] = w.take<uint16_t>(packed_weight_elems(s.Nqkv(), s.d));
      c->pk_o[l] = w.take<uint16_t>(packed_weight_elems(s.d, s.Hq * s.D));
      c->pk_gu[l] = w.take<uint16_t>(packed_weight_elems(2 * s.F, s.d));
      c->pk_down[l] = w.take<uint16_t>(packed_weight_elems(s.d, s.F));
    }
    c->pk_lm = w.take<uint16_t>(packed_weight_elems(s.V, s.d));
  }
  return (w.off + 255) & ~(size_t)255;
}

void fill_shape(bs_ctx* c, const bs_model_desc* d, int B_max, int k_max) {
  c->s = Shape{d->n_layers, d->d_model, d->n_q_heads, d->n_kv_heads, d->head_dim, d->d_ffn, d->vocab, d->dtype,
               d->rms_eps, d->rope_theta};
  c->B_max = B_max;
  c->k_max = k_max;
  c->M_max = B_max * (k_max + 1);
}

bs_status fail(bs_ctx* c, bs_status st, const char* msg) {
  if (c) c->err = msg;
  return st;
}

// RAII-less helper: records an event pair around one launch when its class is being profiled.
struct ProfScope {
  bs_ctx* c; hipStream_t st; bool on; hipEvent_t stop;
  ProfScope(bs_ctx* c_, int cls, hipStream_t st_) : c(c_), st(st_), on(false), stop(nullptr) {
    if (c->prof_class != cls || c->prof_used + 2 > 8192) return;
    if (c->prof_ev.size() < c->prof_used + 2) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
      c->prof_ev.push_back(a);
      c->prof_ev.push_back(b);
    }
    hipEvent_t start = c->prof_ev[c->prof_used];
    stop = c->prof_ev[c->prof_used + 1];
    c->prof_used += 2;
    (void)hipEventRecord(start, st);
    on = true;
  }
  ~ProfScope() { if (on) (void)hipEventRecord(stop, st); }
};

bs_status check_hip(bs_ctx* c) {
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) return BS_OK;
  c->err = std::string("HIP: ") + hipGetErrorString(e);
  return BS_EHIP;
}

}  // namespace

// Called by launch_attention around its main kernel when attention is the profiled class.
void attention_prof_mark(void* token, hipStream_t st, bool begin) {
  bs_ctx* c = (bs_ctx*)token;
  if (begin) {
    ProfScope s(c, BS_PROF_ATTENTION, st);
    c->prof_pending_stop = s.on ? s.stop : nullptr;
    s.on = false;                       // the stop event is recorded by the matching end mark
  } else if (c->prof_pending_stop) {
    (void)hipEventRecord(c->prof_pending_stop, st);
    c->prof_pending_stop = nullptr;
  }
}

extern "C" {

size_t bs_workspace_bytes(const bs_model_desc* desc, int B_max, int k_max) {
  if (check_desc(desc, B_max, k_max) != BS_OK) return 0;
  bs_ctx tmp;
  fill_shape(&tmp, desc, B_max, k_max);
  return carve(&tmp, nullptr);
}

bs_status bs_create(const bs_model_desc* desc, const bs_weights* w, const bs_kv_desc* kv, void* workspace,
                    size_t workspace_bytes, int B_max, int k_max, void* stream, bs_ctx** out) {
  if (!out) return BS_EINVAL;
  *out = nullptr;
  if (!desc || !w || !kv || !workspace) return BS_EINVAL;
  bs_status st = check_desc(desc, B_max, k_max);
  if (st != BS_OK) return st;
  if (!w->embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wqkv || !w->wo || !w->mlp_norm ||
      !w->w_gate_up || !w->w_down)
    return BS_EINVAL;
  if (!kv->k_pages || !kv->v_pages || !kv->block_table || !kv->ctx_len) return BS_EINVAL;
  if (kv->n_pages < 1 || kv->n_slots < 1 || kv->max_pages_per_seq < 1) return BS_ESHAPE;
  if (((uintptr_t)workspace & 255) != 0) return BS_EINVAL;
  bs_ctx* c = new (std::nothrow) bs_ctx();
  if (!c) return BS_EINVAL;
  fill_shape(c, desc, B_max, k_max);
  if (carve(c, nullptr) > workspace_bytes) { delete c; return BS_ECAPACITY; }
  carve(c, (char*)workspace);
  const int L = desc->n_layers;
  launch_clear_status(c->plan.status, (hipStream_t)stream);   // before the packing kernels, which may set BS_FAULT_RANGE
  for (int l = 0; l < L; ++l) {
    if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->mlp_norm[l] || !w->w_gate_up[l] || !w->w_down[l] ||
        !kv->k_pages[l] || !kv->v_pages[l]) { delete c; return BS_EINVAL; }
    c->attn_norm.push_back(w->attn_norm[l]);
    c->mlp_norm.push_back(w->mlp_norm[l]);
    if (desc->dtype == BS_F32) {
      c->wqkv.push_back(w->wqkv[l]);
      c->wo.push_back(w->wo[l]);
      c->w_gate_up.push_back(w->w_gate_up[l]);
      c->w_down.push_back(w->w_down[l]);
    } else {       // one-time re-pack into MFMA operand order (float16); the originals are not used afterwards
      const Shape& s = c->s;
      hipStream_t ps = (hipStream_t)stream;
      launch_pack_weight(w->wqkv[l], s.Nqkv(), s.d, c->pk_qkv[l], c->plan.status, ps);
      launch_pack_weight(w->wo[l], s.d, s.Hq * s.D, c->pk_o[l], c->plan.status, ps);
      launch_pack_weight(w->w_gate_up[l], 2 * s.F, s.d, c->pk_gu[l], c->plan.status, ps);
      launch_pack_weight(w->w_down[l], s.d, s.F, c->pk_down[l], c->plan.status, ps);
      c->wqkv.push_back(c->pk_qkv[l]);
      c->wo.push_back(c->pk_o[l]);
      c->w_gate_up.push_back(c->pk_gu[l]);
      c->w_down.push_back(c->pk_down[l]);
    }
    c->k_pages.push_back(kv->k_pages[l]);
    c->v_pages.push_back(kv->v_pages[l]);
  }
  c->embed = w->embed;
  c->lm_head = w->lm_head;
  if (desc->dtype == BS_BF16) {
    launch_pack_weight(w->lm_head, desc->vocab, desc->d_model, c->pk_lm, c->plan.status, (hipStream_t)stream);
    c->lm_head = c->pk_lm;
  }
  c->final_norm = w->final_norm;
  c->kv = KvView{kv->n_pages, kv->n_slots, kv->max_pages_per_seq, kv->block_table, kv->ctx_len};
  launch_rope_table(c->s, c->inv_freq, (hipStream_t)stream);
  launch_attention_init(c->s, c->B_max, c->attn_scratch, (hipStream_t)stream);
  st = check_hip(c);
  if (st != BS_OK) { bs_destroy(c); return st; }
  *out = c;
  return BS_OK;
}

void bs_destroy(bs_ctx* ctx) {
  if (!ctx) return;
  for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
  delete ctx;
}

bs_status bs_profile_begin(bs_ctx* c, int kernel_class) {
  if (!c) return BS_EINVAL;
  if (kernel_class < BS_PROF_NONE || kernel_class > BS_PROF_EMPTY) return fail(c, BS_EINVAL, "bs_profile_begin: unknown class");
  c->prof_class = kernel_class;
  c->prof_used = 0;
  return BS_OK;
}

bs_status bs_profile_end(bs_ctx* c, void* stream, float* total_ms, int* launches) {
  if (!c || !total_ms || !launches) return BS_EINVAL;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return check_hip(c);
  float tot = 0.f;
  for (size_t i = 0; i + 1 < c->prof_used; i += 2) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->prof_ev[i], c->prof_ev[i + 1]) != hipSuccess) return check_hip(c);
    tot += ms;
  }
  *total_ms = tot;
  *launches = (int)(c->prof_used / 2);
  c->prof_class = BS_PROF_NONE;
  c->prof_used = 0;
  return BS_OK;
}

const char* bs_last_error(const bs_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

bs_status bs_pool_bind(bs_ctx* c, int n_prompts, int n_rollouts, const int32_t* pool_tokens,
                       const int64_t* rollout_offsets, const int32_t* prompt_rollout_begin) {
  if (!c) return BS_EINVAL;
  if (n_prompts < 1 || n_rollouts < 0 || !pool_tokens || !rollout_offsets || !prompt_rollout_begin)
    return fail(c, BS_EINVAL, "bs_pool_bind: null pointer or bad count");
  c->n_prompts = n_prompts;
  c->n_rollouts = n_rollouts;
  c->pool_tokens = pool_tokens;
  c->rollout_offsets = rollout_offsets;
  c->prompt_rollout_begin = prompt_rollout_begin;
  return BS_OK;
}

bs_status bs_index_bind(bs_ctx* c, const void* blob_host, const void* blob_dev, size_t bytes) {
  if (!c) return BS_EINVAL;
  if (!blob_host && !blob_dev) { c->index_blob = nullptr; c->index_prompts = 0; return BS_OK; }
  int np = 0;
  if (!blob_host || !blob_dev || !index_header_ok((const int32_t*)blob_host, bytes, &np))
    return fail(c, BS_EINVAL, "bs_index_bind: not a blob of bs_index_build, or size mismatch");
  if (((uintptr_t)blob_dev & 3) != 0) return fail(c, BS_EINVAL, "bs_index_bind: device copy must be 4-byte aligned");
  c->index_blob = (const int32_t*)blob_dev;
  c->index_prompts = np;
  return BS_OK;
}

bs_status bs_draft_lookup(bs_ctx* c, int B, const int32_t* seq_prompt, const int32_t* tail_tokens, int max_match,
                          int min_match, int k_max, int32_t* draft_tokens, int32_t* draft_len, void* stream) {
  if (!c) return BS_EINVAL;
  if (!c->pool_tokens && !c->index_blob) return fail(c, BS_ESTATE, "bs_draft_lookup: no pool or index bound");
  if (!seq_prompt || !tail_tokens || !draft_tokens || !draft_len) return fail(c, BS_EINVAL, "bs_draft_lookup: null pointer");
  if (B < 1 || B > c->B_max || k_max < 0 || k_max > c->k_max || max_match < 1 || max_match > 8 || min_match < 1 ||
      min_match > max_match)
    return fail(c, BS_ESHAPE, "bs_draft_lookup: B, k_max or match lengths out of range");
  ProfScope ps(c, BS_PROF_LOOKUP, (hipStream_t)stream);
  if (c->index_blob) {
    launch_index_lookup(c->index_blob, c->index_prompts, seq_prompt, tail_tokens, B, max_match, min_match, k_max,
                        draft_tokens, draft_len, (hipStream_t)stream);
    return check_hip(c);
  }
  launch_lookup(B, c->n_prompts, c->pool_tokens, c->rollout_offsets, c->prompt_rollout_begin, seq_prompt, tail_tokens,
                max_match, min_match, k_max, draft_tokens, draft_len, (hipStream_t)stream);
  return check_hip(c);
}

bs_status bs_verify_step(bs_ctx* c, int B, const int32_t* seq_slot, const int32_t* last_token,
                         const int32_t* draft_tokens, const int32_t* draft_len, int k_max, float* logits_debug,
                         void* stream) {
  if (!c) return BS_EINVAL;
  if (!seq_slot || !last_token || !draft_len || (k_max > 0 && !draft_tokens))
    return fail(c, BS_EINVAL, "bs_verify_step: null pointer");
  if (B < 1 || B > c->B_max || k_max < 0 || k_max > c->k_max)
    return fail(c, BS_ESHAPE, "bs_verify_step: B or k_max exceeds the context's limits");
  hipStream_t st = (hipStream_t)stream;
  const Shape& s = c->s;
  const int M_max = B * (k_max + 1);
  const Plan& p = c->plan;
  int attn_s_min, attn_force;
  attention_plan_params(s, B, k_max, &attn_s_min, &attn_force);
  launch_plan(p, c->kv, B, k_max, s.V, seq_slot, last_token, draft_tokens, draft_len, true, attn_s_min, attn_force, s.L, st);
  launch_embed(s, p, M_max, c->embed, c->h, c->inv_freq, c->rope_cos, c->rope_sin, st);
  const bool slab_mode = s.dtype == BS_BF16;   // float32 epilogues go through K-split slabs (see gemm.hip)
  SlabRule pending{0, 0, 0, 0, 0};              // slabs of the last residual projection not yet added to h
  for (int l = 0; l < s.L; ++l) {
    { ProfScope ps(c, BS_PROF_EMPTY, st); }
    launch_rmsnorm(s, p, M_max, c->h, c->slabs, pending, c->attn_norm[l], c->a, st);
    if (qkv_rope_supported(s) && !c->unfused_qkv) {
      ProfScope ps(c, BS_PROF_GEMM_QKV, st);
      launch_qkv_rope(s, p, c->kv, M_max, c->a, c->wqkv[l], c->rope_cos, c->rope_sin, c->q, c->k_pages[l], c->v_pages[l], st);
    } else {
      int nq;
      { ProfScope ps(c, BS_PROF_GEMM_QKV, st);
        nq = launch_gemm(s.dtype, EPI_STORE_F32, p.n_rows, M_max, s.Nqkv(), s.d, c->a, nullptr, c->wqkv[l],
                         slab_mode ? (void*)c->slabs : (void*)c->qkv, p.status, st); }
      launch_rope_append(s, p, c->kv, M_max, c->rope_cos, c->rope_sin, slab_mode ? c->slabs : c->qkv, nq > 0 ? nq : 1, c->q,
                         c->k_pages[l], c->v_pages[l], st);
    }
    launch_attention(s, p, c->kv, l, B, c->B_max, k_max, M_max, c->q, c->k_pages[l], c->v_pages[l], c->attn_out, c->attn_scratch,
                     c->prof_class == BS_PROF_ATTENTION ? (void*)c : nullptr, st);
    { ProfScope ps(c, BS_PROF_GEMM_O, st);
      pending = launch_gemm_resid(s.dtype, p.n_rows, M_max, s.d, s.Hq * s.D, c->attn_out, c->wo[l],
                                  slab_mode ? (void*)c->slabs : (void*)c->h, p.status, st); }
    launch_rmsnorm(s, p, M_max, c->h, c->slabs, pending, c->mlp_norm[l], c->a, st);
    { ProfScope ps(c, BS_PROF_GEMM_GATE_UP, st);
      launch_gemm(s.dtype, EPI_SWIGLU, p.n_rows, M_max, s.F, s.d, c->a, nullptr, c->w_gate_up[l], c->act, p.status, st); }
    { ProfScope ps(c, BS_PROF_GEMM_DOWN, st);
      pending = launch_gemm_resid(s.dtype, p.n_rows, M_max, s.d, s.F, c->act, c->w_down[l],
                                  slab_mode ? (void*)c->slabs : (void*)c->h, p.status, st); }
  }
  launch_rmsnorm(s, p, M_max, c->h, c->slabs, pending, c->final_norm, c->hf, st);
  if (logits_debug && s.dtype == BS_F32)
    launch_gemm(s.dtype, EPI_STORE_F32, p.n_rows, M_max, s.V, s.d, c->hf, nullptr, c->lm_head, logits_debug, p.status, st);
  if (logits_debug && s.dtype == BS_BF16) {
    // same kernel and loop order as the fused path of bs_accept_resample, so the values are identical
    launch_lmhead_stats(s, p, M_max, c->hf, c->lm_head, 1.0f, c->sb, logits_debug, st);
  }
  c->verify_pending = true;
  c->last_B = B;
  c->last_k_max = k_max;
  return check_hip(c);
}

static bs_status accept_common(bs_ctx* c, int B, int V, const float* given_logits, const int32_t* draft_tokens,
                               const int32_t* draft_len, int k_max, const void* q_logits, int q_dtype, float temperature,
                               int eos_id, int emit_bonus, const float* u_accept, const float* u_sample,
                               int32_t* n_accepted, int32_t* out_tokens, int32_t* n_emitted, uint32_t* near_tie,
                               hipStream_t st) {
  const Shape& s = c->s;
  const Plan& p = c->plan;
  const int M_max = B * (k_max + 1);
  const float inv_temp = temperature > 0.f ? 1.0f / temperature : 1.0f;
  const float* sample_base;
  bool rows_selected = false;
  int n_vtiles;
  // top-k / top-p act on a sampled distribution only; they need every row's float32 logits in memory
  FilterArgs filter{0, c->top_k, c->top_p, nullptr, V};
  filter.on = (temperature > 0.f && ((c->top_k > 0 && c->top_k < V) || c->top_p < 1.0f)) ? 1 : 0;
  if (filter.on && V > kFilterMaxVocab) return fail(c, BS_ESHAPE, "accept_resample: top-k / top-p support at most 262136 vocabulary entries");
  if (filter.on && !given_logits && s.dtype == BS_BF16 && !c->filter_logits)
    return fail(c, BS_ESTATE, "accept_resample: top-k / top-p on a bf16 model need the logits scratch of bs_set_filter");
  if (given_logits) launch_plan(p, c->kv, B, k_max, V, nullptr, nullptr, draft_tokens, draft_len, false, 0, 0, 0, st);
  if (given_logits) {
    launch_logit_stats(p, M_max, V, given_logits, inv_temp, c->sb, st);
    n_vtiles = (V + 1023) / 1024;
    sample_base = given_logits;
  } else if (s.dtype == BS_F32) {
    launch_gemm(s.dtype, EPI_STORE_F32, p.n_rows, M_max, s.V, s.d, c->hf, nullptr, c->lm_head, c->full_logits, p.status, st);
    launch_logit_stats(p, M_max, V, c->full_logits, inv_temp, c->sb, st);
    n_vtiles = (V + 1023) / 1024;
    sample_base = c->full_logits;
  } else {
    { ProfScope ps(c, BS_PROF_LMHEAD, st);
      launch_lmhead_stats(s, p, M_max, c->hf, c->lm_head, inv_temp, c->sb, filter.on ? c->filter_logits : nullptr, st); }
    n_vtiles = (V + 63) / 64;
    if (filter.on) {
      sample_base = c->filter_logits;                  // every row is in memory: no second LM-head pass
    } else {
      sample_base = c->sb.sel_logits;
      rows_selected = true;
    }
  }
  filter.logits = sample_base;
  // (Running these HBM-bound statistics on a second stream beside the MFMA-bound LM-head pass was measured: the
  // step got 2 % slower, every kernel of the process paying about 1 us more once a second stream exists.)
  if (q_logits) launch_q_stats(p, M_max, V, q_logits, q_dtype, c->sb, st);
  launch_accept_scan(p, B, k_max, M_max, n_vtiles, q_logits != nullptr, temperature, eos_id, emit_bonus, u_accept, c->sb,
                     filter, n_accepted, out_tokens, n_emitted, near_tie, st);
  if (temperature > 0.f) {
    if (rows_selected) launch_lmhead_rows(s, B, c->hf, c->lm_head, c->sb, st);
    ProfScope ps(c, BS_PROF_SAMPLE, st);
    launch_sample(B, k_max, V, sample_base, rows_selected, q_logits, q_dtype, temperature, filter.on != 0, u_sample, c->sb,
                  n_accepted, out_tokens, n_emitted, near_tie, st);
  }
  return check_hip(c);
}

static bs_status check_accept_args(bs_ctx* c, int B, const int32_t* draft_tokens, const int32_t* draft_len, int k_max,
                                   const void* q_logits, int q_dtype, float temperature, const float* u_accept,
                                   const float* u_sample, int32_t* n_accepted, int32_t* out_tokens, int32_t* n_emitted,
                                   uint32_t* near_tie) {
  if (!draft_len || (k_max > 0 && (!draft_tokens || !u_accept)) || !u_sample || !n_accepted || !out_tokens ||
      !n_emitted || !near_tie)
    return fail(c, BS_EINVAL, "accept_resample: null pointer");
  if (!(temperature >= 0.f)) return fail(c, BS_EINVAL, "accept_resample: temperature must be >= 0");
  if (q_logits && q_dtype != BS_F32 && q_dtype != BS_BF16) return fail(c, BS_EINVAL, "accept_resample: bad q_dtype");
  if (B < 1 || B > c->B_max || k_max < 0 || k_max > c->k_max)
    return fail(c, BS_ESHAPE, "accept_resample: B or k_max exceeds the context's limits");
  return BS_OK;
}

bs_status bs_accept_resample(bs_ctx* c, int B, const int32_t* draft_tokens, const int32_t* draft_len, int k_max,
                             const void* q_logits, int q_dtype, float temperature, int eos_id, int emit_bonus,
                             const float* u_accept, const float* u_sample, int32_t* n_accepted, int32_t* out_tokens,
                             int32_t* n_emitted, uint32_t* near_tie, void* stream) {
  if (!c) return BS_EINVAL;
  bs_status st = check_accept_args(c, B, draft_tokens, draft_len, k_max, q_logits, q_dtype, temperature, u_accept,
                                   u_sample, n_accepted, out_tokens, n_emitted, near_tie);
  if (st != BS_OK) return st;
  if (!c->verify_pending) return fail(c, BS_ESTATE, "bs_accept_resample: no verify step pending");
  if (B != c->last_B || k_max != c->last_k_max)
    return fail(c, BS_ESHAPE, "bs_accept_resample: B / k_max differ from the verify step");
  return accept_common(c, B, c->s.V, nullptr, draft_tokens, draft_len, k_max, q_logits, q_dtype, temperature, eos_id,
                       emit_bonus, u_accept, u_sample, n_accepted, out_tokens, n_emitted, near_tie, (hipStream_t)stream);
}

bs_status bs_accept_resample_logits(bs_ctx* c, int B, int vocab, const float* logits, const int32_t* draft_tokens,
                                    const int32_t* draft_len, int k_max, const void* q_logits, int q_dtype,
                                    float temperature, int eos_id, int emit_bonus, const float* u_accept,
                                    const float* u_sample, int32_t* n_accepted, int32_t* out_tokens, int32_t* n_emitted,
                                    uint32_t* near_tie, void* stream) {
  if (!c) return BS_EINVAL;
  if (!logits) return fail(c, BS_EINVAL, "bs_accept_resample_logits: null logits");
  if (vocab < 2 || vocab > c->s.V) return fail(c, BS_ESHAPE, "bs_accept_resample_logits: vocab outside [2, model vocab]");
  bs_status st = check_accept_args(c, B, draft_tokens, draft_len, k_max, q_logits, q_dtype, temperature, u_accept,
                                   u_sample, n_accepted, out_tokens, n_emitted, near_tie);
  if (st != BS_OK) return st;
  c->verify_pending = false;      // the plan in the workspace now describes this call, not a verify step
  return accept_common(c, B, vocab, logits, draft_tokens, draft_len, k_max, q_logits, q_dtype, temperature, eos_id,
                       emit_bonus, u_accept, u_sample, n_accepted, out_tokens, n_emitted, near_tie, (hipStream_t)stream);
}

bs_status bs_set_filter(bs_ctx* c, int top_k, float top_p, float* logits_scratch) {
  if (!c) return BS_EINVAL;
  if (!(top_p > 0.f)) return fail(c, BS_EINVAL, "bs_set_filter: top_p must be in (0, 1] (>= 1 switches it off)");
  c->top_k = top_k > 0 ? top_k : 0;
  c->top_p = top_p < 1.0f ? top_p : 1.0f;
  c->filter_logits = logits_scratch;
  return BS_OK;
}

bs_status bs_kv_commit(bs_ctx* c, int B, const int32_t* seq_slot, const int32_t* n_commit, void* stream) {
  if (!c) return BS_EINVAL;
  if (!seq_slot || !n_commit) return fail(c, BS_EINVAL, "bs_kv_commit: null pointer");
  if (!c->verify_pending) return fail(c, BS_ESTATE, "bs_kv_commit: no verify step pending");
  if (B != c->last_B) return fail(c, BS_ESHAPE, "bs_kv_commit: B differs from the verify step");
  launch_commit(c->plan, c->kv, B, seq_slot, n_commit, (hipStream_t)stream);
  c->verify_pending = false;
  return check_hip(c);
}

bs_status bs_kv_lengths(bs_ctx* c, int B, const int32_t* seq_slot, int32_t* ctx_len_out, void* stream) {
  if (!c) return BS_EINVAL;
  if (!seq_slot || !ctx_len_out) return fail(c, BS_EINVAL, "bs_kv_lengths: null pointer");
  if (B < 1) return fail(c, BS_ESHAPE, "bs_kv_lengths: B must be positive");
  launch_kv_lengths(c->kv, B, seq_slot, ctx_len_out, c->plan.status, (hipStream_t)stream);
  return check_hip(c);
}

static bs_status kv_copy(bs_ctx* c, int layer, int slot, int pos0, int n, void* k_rows, void* v_rows, bool to_pages,
                         void* stream) {
  if (!c) return BS_EINVAL;
  if (!k_rows || !v_rows) return fail(c, BS_EINVAL, "bs_kv_write/read: null pointer");
  if (layer < 0 || layer >= c->s.L || slot < 0 || slot >= c->kv.n_slots || pos0 < 0 || n < 0)
    return fail(c, BS_ESHAPE, "bs_kv_write/read: layer, slot or range out of bounds");
  if ((long)pos0 + n > (long)c->kv.max_pages * kPage) return fail(c, BS_ECAPACITY, "bs_kv_write/read: beyond the slot's pages");
  launch_kv_copy(c->s, c->kv, slot, pos0, n, c->k_pages[layer], c->v_pages[layer], k_rows, v_rows, to_pages,
                 c->plan.status, (hipStream_t)stream);
  return check_hip(c);
}

bs_status bs_kv_write(bs_ctx* c, int layer, int slot, int pos0, int n, const void* k_rows, const void* v_rows,
                      void* stream) {
  return kv_copy(c, layer, slot, pos0, n, (void*)k_rows, (void*)v_rows, true, stream);
}
bs_status bs_kv_read(bs_ctx* c, int layer, int slot, int pos0, int n, void* k_rows, void* v_rows, void* stream) {
  return kv_copy(c, layer, slot, pos0, n, k_rows, v_rows, false, stream);
}

bs_status bs_poll_status(bs_ctx* c, void* stream, int32_t* fault_out) {
  if (!c || !fault_out) return BS_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  int32_t host = 0;
  if (hipMemcpyAsync(&host, c->plan.status, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess)
    return check_hip(c) == BS_OK ? fail(c, BS_EHIP, "bs_poll_status: copy failed") : BS_EHIP;
  launch_clear_status(c->plan.status, st);
  *fault_out = host;
  return check_hip(c);
}

// ---------------------------------------------------------------------------------------------------------------
// Allocation-free variant of bs_accept_resample_logits (see the header).  Everything the sampler kernels keep
// between launches (the device plan of the packed rows, per-tile and per-row softmax statistics, the float64
// sampling partials) lives in g_noalloc_scratch, a file-scope device array, instead of a caller-supplied workspace.
// The array's name is only a host-side handle: its device address is obtained once per device with
// hipGetSymbolAddress and that address is what is carved and handed to the kernels.
constexpr int kNoAllocMaxB = 1024;                       // sequences per call
constexpr int kNoAllocMaxRows = 2048;                    // packed rows B * (k_max + 1) per call
constexpr int kNoAllocMaxVocab = 262144;
constexpr size_t kNoAllocScratchBytes = (size_t)9 << 20; // 9 MiB per device, held until the process ends
constexpr int kNoAllocMaxDevices = 64;
static __device__ __align__(256) unsigned char g_noalloc_scratch[kNoAllocScratchBytes];

namespace {
struct NoAllocState {
  bs_ctx* ctx = nullptr;       // host-side view of this device's copy of the array (never freed)
};
NoAllocState g_noalloc[kNoAllocMaxDevices];
std::mutex g_noalloc_mutex;

// Host-side view of the current device's scratch array, created at the first call on that device.
bs_status noalloc_state(bs_ctx** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kNoAllocMaxDevices) return BS_EHIP;
  std::lock_guard<std::mutex> lock(g_noalloc_mutex);
  if (!g_noalloc[dev].ctx) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_noalloc_scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return BS_EHIP;
    }
    bs_ctx* c = new (std::nothrow) bs_ctx();
    if (!c) return BS_ECAPACITY;
    c->s = Shape{1, 64, 1, 1, 64, 64, kNoAllocMaxVocab, BS_F32, 1e-6f, 1e6f};   // only V and dtype are consulted
    c->B_max = kNoAllocMaxB;
    c->k_max = BS_MAX_K;
    c->M_max = kNoAllocMaxRows;
    c->kv = KvView{0, 0, 0, nullptr, nullptr};
    for (int pass = 0; pass < 2; ++pass) {               // measure, then lay out
      Carver w{pass ? (char*)ptr : nullptr};
      carve_plan(w, c->plan, kNoAllocMaxB, kNoAllocMaxRows, false, 0);
      carve_sampler(w, c->sb, kNoAllocMaxB, kNoAllocMaxRows, (kNoAllocMaxVocab + 1023) / 1024);
      if (w.off > kNoAllocScratchBytes) { delete c; return BS_ECAPACITY; }
    }
    g_noalloc[dev].ctx = c;
  }
  *out = g_noalloc[dev].ctx;
  return BS_OK;
}
}  // namespace

bs_status bs_accept_resample_logits_noalloc(int B, int vocab, const float* logits, const int32_t* draft_tokens,
                                            const int32_t* draft_len, int k_max, const void* q_logits, int q_dtype,
                                            float temperature, int eos_id, int emit_bonus, const float* u_accept,
                                            const float* u_sample, int32_t* n_accepted, int32_t* out_tokens,
                                            int32_t* n_emitted, uint32_t* near_tie, void* stream) {
  if (!logits || !draft_len || (k_max > 0 && (!draft_tokens || !u_accept)) || !u_sample || !n_accepted || !out_tokens ||
      !n_emitted || !near_tie)
    return BS_EINVAL;
  if (!(temperature >= 0.f)) return BS_EINVAL;
  if (q_logits && q_dtype != BS_F32 && q_dtype != BS_BF16) return BS_EINVAL;
  if (B < 1 || B > kNoAllocMaxB || k_max < 0 || k_max > BS_MAX_K || (long)B * (k_max + 1) > kNoAllocMaxRows ||
      vocab < 2 || vocab > kNoAllocMaxVocab)
    return BS_ESHAPE;                                    // beyond the fixed maximum of the static scratch
  bs_ctx* c = nullptr;
  const bs_status st = noalloc_state(&c);
  if (st != BS_OK) return st;
  // The array keeps the previous call's contents.  The only word a call relies on being zero is the status word
  // (the plan and the statistics are written before they are read); it is cleared by a kernel, not a memset node,
  // so that the call can be captured into a HIP graph.
  launch_clear_status(c->plan.status, (hipStream_t)stream);
  return accept_common(c, B, vocab, logits, draft_tokens, draft_len, k_max, q_logits, q_dtype, temperature, eos_id,
                       emit_bonus, u_accept, u_sample, n_accepted, out_tokens, n_emitted, near_tie, (hipStream_t)stream);
}

// Not part of the public ABI: selects the unfused QKV path (projection GEMM, then the rotary / append kernel)
// for models that would use the fused kernel, so that tests cover both.
void bs_debug_unfused_qkv(bs_ctx* c, int on) { if (c) c->unfused_qkv = on != 0; }

// Not part of the public ABI: address of an intermediate buffer of the last verify step, for
// kernel-level debugging (0 h, 1 normed rows, 2 qkv f32, 3 q, 4 attention out, 5 mlp act, 6 final rows), or of
// the last accept step (7, 8, 9: per-row filter threshold key, index cut, log of the kept mass).
void* bs_debug_buffer(bs_ctx* c, int which) {
  if (!c) return nullptr;
  switch (which) {
    case 0: return c->h;
    case 1: return c->a;
    case 2: return c->qkv;
    case 3: return c->q;
    case 4: return c->attn_out;
    case 5: return c->act;
    case 6: return c->hf;
    case 7: return c->sb.f_key;
    case 8: return c->sb.f_idx;
    case 9: return c->sb.f_lse;
    default: return nullptr;
  }
}

// Not part of the public ABI: copies the first `bytes` bytes of a bs_debug_buffer to a device buffer of the caller.
int bs_debug_copy(bs_ctx* c, int which, void* dst, size_t bytes, void* stream) {
  void* src = bs_debug_buffer(c, which);
  if (!src || !dst) return BS_EINVAL;
  return hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream) == hipSuccess ? BS_OK : BS_EHIP;
}

}  // extern "C"
