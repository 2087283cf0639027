"""Torch plumbing around the C ABI: device allocations (weights, paged KV cache, block table,
workspace) and tensor-level wrappers of the step calls.  No arithmetic of the method lives here;
every step runs in libbubblespec.so."""
import torch

from . import binding as B

TORCH_DTYPE = {B.BS_F32: torch.float32, B.BS_BF16: torch.bfloat16}


def fuse_weights(w, dtype, device):
    """Layout marshalling: per-matrix weights (oracle naming: wq/wk/wv, w_gate/w_up, ...) as torch tensors
    -> the fused row-major layout of bs_weights on `device`."""
    td = TORCH_DTYPE[dtype]
    dev = lambda t, dt=td: t.to(device=device, dtype=dt).contiguous()
    out = {"embed": dev(w["embed"]), "lm_head": dev(w["lm_head"]), "final_norm": dev(w["final_norm"], torch.float32),
           "attn_norm": [], "wqkv": [], "wo": [], "mlp_norm": [], "w_gate_up": [], "w_down": []}
    for lw in w["layers"]:
        out["attn_norm"].append(dev(lw["attn_norm"], torch.float32))
        out["mlp_norm"].append(dev(lw["mlp_norm"], torch.float32))
        out["wqkv"].append(torch.cat([dev(lw["wq"]), dev(lw["wk"]), dev(lw["wv"])], dim=0).contiguous())
        out["wo"].append(dev(lw["wo"]))
        out["w_gate_up"].append(torch.cat([dev(lw["w_gate"]), dev(lw["w_up"])], dim=0).contiguous())
        out["w_down"].append(dev(lw["w_down"]))
    return out


class Engine:
    """Owns the device buffers of one context and forwards to the C ABI."""

    def __init__(self, desc, weights, n_slots, max_ctx, B_max, k_max, device="cuda:0", page_perm_seed=None,
                 slot_tokens=None):
        """max_ctx: token capacity of every slot; slot_tokens (optional, one entry per slot) gives every slot its own
        capacity instead, so that a ragged batch only takes the pages it needs (block-table entries beyond a slot's
        pages are -1)."""
        self.desc = dict(desc)
        self.device = torch.device(device)
        self.cdesc = B.make_desc(desc)
        self.B_max, self.k_max = B_max, k_max
        self.weights = weights
        # page encoding: float32 models store float32; bf16 models store bf16-rounded values as float16 bits
        td = torch.float32 if desc["dtype"] == B.BS_F32 else torch.float16
        P = B.BS_PAGE_TOKENS
        caps = [int(max_ctx)] * n_slots if slot_tokens is None else [int(t) for t in slot_tokens]
        assert len(caps) == n_slots
        pages_of = [(c + P - 1) // P for c in caps]
        self.max_pages = max(pages_of)
        self.n_slots = n_slots
        self.n_pages = sum(pages_of)
        page_elems = desc["n_kv_heads"] * P * desc["head_dim"]
        # pages are zero-initialised: masked positions still enter the P*V product with weight 0
        self.k_pages = [torch.zeros(self.n_pages, page_elems, dtype=td, device=self.device)
                        for _ in range(desc["n_layers"])]
        self.v_pages = [torch.zeros(self.n_pages, page_elems, dtype=td, device=self.device)
                        for _ in range(desc["n_layers"])]
        ids = torch.arange(self.n_pages, dtype=torch.int32)
        if page_perm_seed is not None:      # scatter pages to exercise the block table
            g = torch.Generator().manual_seed(page_perm_seed)
            ids = ids[torch.randperm(self.n_pages, generator=g)]
        table = torch.full((n_slots, self.max_pages), -1, dtype=torch.int32)
        at = 0
        for b, n in enumerate(pages_of):
            table[b, :n] = ids[at:at + n]
            at += n
        self.block_table = table.contiguous().to(self.device)
        self.ctx_len = torch.zeros(n_slots, dtype=torch.int32, device=self.device)
        nbytes = B.bs_workspace_bytes(self.cdesc, B_max, k_max)
        if nbytes == 0:
            raise B.BsError(B.BS_ESHAPE, "bs_workspace_bytes rejected the shape")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        kv = dict(n_pages=self.n_pages, n_slots=n_slots, max_pages_per_seq=self.max_pages, k_pages=self.k_pages,
                  v_pages=self.v_pages, block_table=self.block_table, ctx_len=self.ctx_len)
        self.ctx = B.bs_create(self.cdesc, weights, kv, self.workspace, B_max, k_max)
        self._pool = None

    def close(self):
        if self.ctx is not None:
            B.bs_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- draft database -----------------------------------------------------------------------
    def pool_bind(self, pool_tokens, rollout_offsets, prompt_rollout_begin):
        self._pool = (pool_tokens.to(self.device, torch.int32).contiguous(),
                      rollout_offsets.to(self.device, torch.int64).contiguous(),
                      prompt_rollout_begin.to(self.device, torch.int32).contiguous())
        B.bs_pool_bind(self.ctx, self._pool[2].numel() - 1, self._pool[1].numel() - 1, *self._pool)

    def index_bind(self, blob_host):
        """Binds a prebuilt index (NumPy blob from binding.bs_index_build); None unbinds and returns to the scan."""
        if blob_host is None:
            self._index = None
            B.bs_index_bind(self.ctx, None, None)
            return
        self._index = (blob_host, torch.from_numpy(blob_host).to(self.device))
        B.bs_index_bind(self.ctx, *self._index)

    def draft_lookup(self, seq_prompt, tail_tokens, max_match, min_match, k_max):
        n = seq_prompt.numel()
        draft_tokens = torch.empty(n, max(k_max, 1), dtype=torch.int32, device=self.device)[:, :k_max].contiguous()
        draft_len = torch.empty(n, dtype=torch.int32, device=self.device)
        B.bs_draft_lookup(self.ctx, n, seq_prompt, tail_tokens, max_match, min_match, k_max, draft_tokens, draft_len)
        return draft_tokens, draft_len

    # -- step ---------------------------------------------------------------------------------
    def verify_step(self, seq_slot, last_token, draft_tokens, draft_len, k_max, want_logits=False):
        n = seq_slot.numel()
        logits = None
        if want_logits:
            logits = torch.zeros(n * (k_max + 1), self.desc["vocab"], dtype=torch.float32, device=self.device)
        B.bs_verify_step(self.ctx, n, seq_slot, last_token, draft_tokens, draft_len, k_max, logits)
        return logits

    def accept_resample(self, draft_tokens, draft_len, k_max, u_accept, u_sample, q_logits=None, temperature=1.0,
                        eos_id=-1, emit_bonus=True, logits=None, vocab=None):
        n = draft_len.numel()
        out = dict(n_accepted=torch.empty(n, dtype=torch.int32, device=self.device),
                   out_tokens=torch.empty(n, k_max + 1, dtype=torch.int32, device=self.device),
                   n_emitted=torch.empty(n, dtype=torch.int32, device=self.device),
                   near_tie=torch.empty(n, dtype=torch.int32, device=self.device))
        q_dtype = B.BS_F32
        if q_logits is not None:
            q_dtype = B.BS_BF16 if q_logits.dtype == torch.bfloat16 else B.BS_F32
        args = (draft_tokens, draft_len, k_max, q_logits, q_dtype, float(temperature), eos_id, emit_bonus, u_accept,
                u_sample, out["n_accepted"], out["out_tokens"], out["n_emitted"], out["near_tie"])
        if logits is None:
            B.bs_accept_resample(self.ctx, n, *args)
        else:
            B.bs_accept_resample_logits(self.ctx, n, vocab if vocab is not None else logits.shape[1], logits, *args)
        return out

    def set_filter(self, top_k=0, top_p=1.0):
        """Top-k / top-p filtering of the target distribution for the following accept steps (0 / 1.0: off).
        bf16 models get the float32 logits scratch the filtered path needs, allocated on first use."""
        on = top_k > 0 or top_p < 1.0
        if on and self.desc["dtype"] == B.BS_BF16 and getattr(self, "_filter_logits", None) is None:
            self._filter_logits = torch.empty(self.B_max * (self.k_max + 1), self.desc["vocab"], dtype=torch.float32,
                                              device=self.device)
        B.bs_set_filter(self.ctx, top_k, top_p, getattr(self, "_filter_logits", None) if on else None)

    def kv_commit(self, seq_slot, n_commit):
        B.bs_kv_commit(self.ctx, seq_slot.numel(), seq_slot, n_commit)

    def kv_lengths(self, seq_slot):
        out = torch.empty(seq_slot.numel(), dtype=torch.int32, device=self.device)
        B.bs_kv_lengths(self.ctx, seq_slot.numel(), seq_slot, out)
        return out

    def kv_write(self, layer, slot, pos0, k_rows, v_rows):
        B.bs_kv_write(self.ctx, layer, slot, pos0, k_rows.shape[0], k_rows.contiguous(), v_rows.contiguous())

    def kv_read(self, layer, slot, pos0, n):
        td = TORCH_DTYPE[self.desc["dtype"]]
        shape = (n, self.desc["n_kv_heads"], self.desc["head_dim"])
        k = torch.empty(shape, dtype=td, device=self.device)
        v = torch.empty(shape, dtype=td, device=self.device)
        B.bs_kv_read(self.ctx, layer, slot, pos0, n, k, v)
        return k, v

    def poll_status(self):
        return B.bs_poll_status(self.ctx)
