"""ctypes binding of libbubblespec.so: one Python function per C entry point, same name, same
argument order (include/bubblespec.h is the contract).  Marshalling only: tensors become raw device
pointers, the current torch stream becomes the hipStream_t.  No computation happens here."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbubblespec.so")

BS_OK, BS_EINVAL, BS_ESHAPE, BS_ECAPACITY, BS_ESTATE, BS_EHIP = range(6)
BS_F32, BS_BF16 = 0, 1
BS_FAULT_DRAFT_LEN, BS_FAULT_KV_PAGES, BS_FAULT_TOKEN_ID, BS_FAULT_COMMIT, BS_FAULT_SLOT, BS_FAULT_RANGE = 1, 2, 4, 8, 16, 32
BS_PAGE_TOKENS = 64
BS_MAX_K = 30
STATUS_NAMES = ["BS_OK", "BS_EINVAL", "BS_ESHAPE", "BS_ECAPACITY", "BS_ESTATE", "BS_EHIP"]

EXPORTS = ["bs_workspace_bytes", "bs_create", "bs_destroy", "bs_last_error", "bs_pool_bind", "bs_draft_lookup",
           "bs_verify_step", "bs_accept_resample", "bs_accept_resample_logits", "bs_kv_commit", "bs_kv_write",
           "bs_kv_read", "bs_poll_status", "bs_profile_begin", "bs_profile_end", "bs_index_build", "bs_index_free",
           "bs_index_bind", "bs_set_filter", "bs_kv_lengths", "bs_accept_resample_logits_noalloc"]
PROF_CLASSES = {"attention": 1, "gemm_qkv": 2, "gemm_o": 3, "gemm_gate_up": 4, "gemm_down": 5, "lmhead": 6,
                "sample": 7, "lookup": 8, "empty": 9}


class bs_model_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("dtype", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class bs_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("attn_norm", C.POINTER(C.c_void_p)), ("wqkv", C.POINTER(C.c_void_p)),
                ("wo", C.POINTER(C.c_void_p)), ("mlp_norm", C.POINTER(C.c_void_p)),
                ("w_gate_up", C.POINTER(C.c_void_p)), ("w_down", C.POINTER(C.c_void_p))]


class bs_kv_desc(C.Structure):
    _fields_ = [("n_pages", C.c_int32), ("n_slots", C.c_int32), ("max_pages_per_seq", C.c_int32),
                ("k_pages", C.POINTER(C.c_void_p)), ("v_pages", C.POINTER(C.c_void_p)),
                ("block_table", C.c_void_p), ("ctx_len", C.c_void_p)]


_lib = None


def lib():
    """Loads the library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libbubblespec.so is not built: run `python -m paper_2605_08862_amd.build` "
                               "(or __graft_entry__.build()) first; there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        vp, i32, f32 = C.c_void_p, C.c_int, C.c_float
        L.bs_workspace_bytes.restype = C.c_size_t
        L.bs_workspace_bytes.argtypes = [C.POINTER(bs_model_desc), i32, i32]
        L.bs_create.argtypes = [C.POINTER(bs_model_desc), C.POINTER(bs_weights), C.POINTER(bs_kv_desc), vp,
                                C.c_size_t, i32, i32, vp, C.POINTER(vp)]
        L.bs_destroy.argtypes = [vp]
        L.bs_destroy.restype = None
        L.bs_last_error.argtypes = [vp]
        L.bs_last_error.restype = C.c_char_p
        L.bs_pool_bind.argtypes = [vp, i32, i32, vp, vp, vp]
        L.bs_index_build.argtypes = [i32, vp, vp, vp, C.POINTER(vp), C.POINTER(C.c_size_t)]
        L.bs_index_free.argtypes = [vp]
        L.bs_index_free.restype = None
        L.bs_index_bind.argtypes = [vp, vp, vp, C.c_size_t]
        L.bs_draft_lookup.argtypes = [vp, i32, vp, vp, i32, i32, i32, vp, vp, vp]
        L.bs_verify_step.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp, vp]
        L.bs_accept_resample.argtypes = [vp, i32, vp, vp, i32, vp, i32, f32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.bs_accept_resample_logits.argtypes = [vp, i32, i32, vp, vp, vp, i32, vp, i32, f32, i32, i32, vp, vp, vp,
                                                vp, vp, vp, vp]
        L.bs_accept_resample_logits_noalloc.argtypes = [i32, i32, vp, vp, vp, i32, vp, i32, f32, i32, i32, vp, vp, vp,
                                                        vp, vp, vp, vp]
        L.bs_set_filter.argtypes = [vp, i32, f32, vp]
        L.bs_kv_commit.argtypes = [vp, i32, vp, vp, vp]
        L.bs_kv_lengths.argtypes = [vp, i32, vp, vp, vp]
        L.bs_kv_write.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
        L.bs_kv_read.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
        L.bs_poll_status.argtypes = [vp, vp, C.POINTER(C.c_int32)]
        L.bs_profile_begin.argtypes = [vp, i32]
        L.bs_profile_end.argtypes = [vp, vp, C.POINTER(C.c_float), C.POINTER(C.c_int)]
        for name in EXPORTS:
            if name not in ("bs_workspace_bytes", "bs_destroy", "bs_last_error", "bs_index_free"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class BsError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__("%s: %s" % (STATUS_NAMES[status] if 0 <= status < 6 else status, msg))
        self.status = status


def _ptr(t):
    """Raw address of a tensor (device or host) or None -> NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous()
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(ctx, st):
    if st != BS_OK:
        msg = lib().bs_last_error(ctx).decode() if ctx else ""
        raise BsError(st, msg)


def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def make_desc(d):
    return bs_model_desc(d["n_layers"], d["d_model"], d["n_q_heads"], d["n_kv_heads"], d["head_dim"], d["d_ffn"],
                         d["vocab"], d["dtype"], d.get("rms_eps", 1e-6), d.get("rope_theta", 1e6))


def bs_workspace_bytes(desc, B_max, k_max):
    return lib().bs_workspace_bytes(C.byref(desc), B_max, k_max)


def bs_create(desc, weights, kv, workspace, B_max, k_max):
    """weights: dict of device tensors (embed, lm_head, final_norm, and lists attn_norm, wqkv, wo, mlp_norm,
    w_gate_up, w_down); kv: dict(n_pages, n_slots, max_pages_per_seq, k_pages[list], v_pages[list],
    block_table, ctx_len).  Returns the opaque context handle."""
    w = bs_weights(weights["embed"].data_ptr(), weights["lm_head"].data_ptr(), weights["final_norm"].data_ptr(),
                   _ptr_array(weights["attn_norm"]), _ptr_array(weights["wqkv"]), _ptr_array(weights["wo"]),
                   _ptr_array(weights["mlp_norm"]), _ptr_array(weights["w_gate_up"]), _ptr_array(weights["w_down"]))
    k = bs_kv_desc(kv["n_pages"], kv["n_slots"], kv["max_pages_per_seq"], _ptr_array(kv["k_pages"]),
                   _ptr_array(kv["v_pages"]), kv["block_table"].data_ptr(), kv["ctx_len"].data_ptr())
    out = C.c_void_p()
    st = lib().bs_create(C.byref(desc), C.byref(w), C.byref(k), workspace.data_ptr(), workspace.numel(), B_max,
                         k_max, _stream(), C.byref(out))
    if st != BS_OK:
        raise BsError(st, "bs_create")
    return out


def bs_destroy(ctx):
    lib().bs_destroy(ctx)


def bs_pool_bind(ctx, n_prompts, n_rollouts, pool_tokens, rollout_offsets, prompt_rollout_begin):
    _check(ctx, lib().bs_pool_bind(ctx, n_prompts, n_rollouts, _ptr(pool_tokens), _ptr(rollout_offsets),
                                   _ptr(prompt_rollout_begin)))


def bs_index_build(pool_tokens, rollout_offsets, prompt_rollout_begin):
    """Host-side index build from NumPy arrays (int32, int64, int32).  Returns the blob as a NumPy int32 array (a
    copy; the library's buffer is released)."""
    import numpy as np
    pt = np.ascontiguousarray(pool_tokens, dtype=np.int32)
    ro = np.ascontiguousarray(rollout_offsets, dtype=np.int64)
    pb = np.ascontiguousarray(prompt_rollout_begin, dtype=np.int32)
    blob, nbytes = C.c_void_p(), C.c_size_t()
    st = lib().bs_index_build(len(pb) - 1, pt.ctypes.data_as(C.c_void_p), ro.ctypes.data_as(C.c_void_p),
                              pb.ctypes.data_as(C.c_void_p), C.byref(blob), C.byref(nbytes))
    if st != BS_OK:
        raise BsError(st, "bs_index_build failed")
    try:
        out = np.frombuffer(C.string_at(blob.value, nbytes.value), dtype=np.int32).copy()
    finally:
        lib().bs_index_free(blob)
    return out


def bs_index_bind(ctx, blob_host, blob_dev):
    """blob_host: NumPy int32 array from bs_index_build (or None to unbind); blob_dev: its device copy (tensor)."""
    if blob_host is None:
        _check(ctx, lib().bs_index_bind(ctx, None, None, 0))
        return
    _check(ctx, lib().bs_index_bind(ctx, blob_host.ctypes.data_as(C.c_void_p), _ptr(blob_dev), blob_host.nbytes))


def bs_draft_lookup(ctx, B, seq_prompt, tail_tokens, max_match, min_match, k_max, draft_tokens, draft_len):
    _check(ctx, lib().bs_draft_lookup(ctx, B, _ptr(seq_prompt), _ptr(tail_tokens), max_match, min_match, k_max,
                                      _ptr(draft_tokens), _ptr(draft_len), _stream()))


def bs_verify_step(ctx, B, seq_slot, last_token, draft_tokens, draft_len, k_max, logits_debug=None):
    _check(ctx, lib().bs_verify_step(ctx, B, _ptr(seq_slot), _ptr(last_token), _ptr(draft_tokens), _ptr(draft_len),
                                     k_max, _ptr(logits_debug), _stream()))


def bs_accept_resample(ctx, B, draft_tokens, draft_len, k_max, q_logits, q_dtype, temperature, eos_id, emit_bonus,
                       u_accept, u_sample, n_accepted, out_tokens, n_emitted, near_tie):
    _check(ctx, lib().bs_accept_resample(ctx, B, _ptr(draft_tokens), _ptr(draft_len), k_max, _ptr(q_logits), q_dtype,
                                         temperature, eos_id, int(emit_bonus), _ptr(u_accept), _ptr(u_sample),
                                         _ptr(n_accepted), _ptr(out_tokens), _ptr(n_emitted), _ptr(near_tie),
                                         _stream()))


def bs_accept_resample_logits(ctx, B, vocab, logits, draft_tokens, draft_len, k_max, q_logits, q_dtype, temperature,
                              eos_id, emit_bonus, u_accept, u_sample, n_accepted, out_tokens, n_emitted, near_tie):
    _check(ctx, lib().bs_accept_resample_logits(ctx, B, vocab, _ptr(logits), _ptr(draft_tokens), _ptr(draft_len),
                                                k_max, _ptr(q_logits), q_dtype, temperature, eos_id, int(emit_bonus),
                                                _ptr(u_accept), _ptr(u_sample), _ptr(n_accepted), _ptr(out_tokens),
                                                _ptr(n_emitted), _ptr(near_tie), _stream()))


def bs_accept_resample_logits_noalloc(B, vocab, logits, draft_tokens, draft_len, k_max, q_logits, q_dtype, temperature,
                                      eos_id, emit_bonus, u_accept, u_sample, n_accepted, out_tokens, n_emitted, near_tie):
    st = lib().bs_accept_resample_logits_noalloc(B, vocab, _ptr(logits), _ptr(draft_tokens), _ptr(draft_len), k_max,
                                                 _ptr(q_logits), q_dtype, temperature, eos_id, int(emit_bonus),
                                                 _ptr(u_accept), _ptr(u_sample), _ptr(n_accepted), _ptr(out_tokens),
                                                 _ptr(n_emitted), _ptr(near_tie), _stream())
    if st != BS_OK:
        raise BsError(st, "bs_accept_resample_logits_noalloc")


def bs_set_filter(ctx, top_k, top_p, logits_scratch):
    _check(ctx, lib().bs_set_filter(ctx, int(top_k), float(top_p), _ptr(logits_scratch)))


def bs_kv_commit(ctx, B, seq_slot, n_commit):
    _check(ctx, lib().bs_kv_commit(ctx, B, _ptr(seq_slot), _ptr(n_commit), _stream()))


def bs_kv_lengths(ctx, B, seq_slot, ctx_len_out):
    _check(ctx, lib().bs_kv_lengths(ctx, B, _ptr(seq_slot), _ptr(ctx_len_out), _stream()))


def bs_kv_write(ctx, layer, slot, pos0, n, k_rows, v_rows):
    _check(ctx, lib().bs_kv_write(ctx, layer, slot, pos0, n, _ptr(k_rows), _ptr(v_rows), _stream()))


def bs_kv_read(ctx, layer, slot, pos0, n, k_rows, v_rows):
    _check(ctx, lib().bs_kv_read(ctx, layer, slot, pos0, n, _ptr(k_rows), _ptr(v_rows), _stream()))


def bs_poll_status(ctx):
    out = C.c_int32(0)
    _check(ctx, lib().bs_poll_status(ctx, _stream(), C.byref(out)))
    return out.value


def bs_profile_begin(ctx, kernel_class):
    _check(ctx, lib().bs_profile_begin(ctx, kernel_class))


def bs_profile_end(ctx):
    ms, n = C.c_float(0), C.c_int(0)
    _check(ctx, lib().bs_profile_end(ctx, _stream(), C.byref(ms), C.byref(n)))
    return ms.value, n.value


def bs_debug_attention_shape(q_blocks=0, n_split=0):
    """Test hook (not part of the public ABI): forces the attention launch shape; 0 = automatic."""
    f = lib().bs_debug_attention_shape
    f.argtypes = [C.c_int, C.c_int]
    f.restype = None
    f(q_blocks, n_split)


def bs_debug_unfused_qkv(ctx, on):
    """Test hook (not part of the public ABI): use the QKV GEMM + separate rotary kernel instead of the fused one."""
    f = lib().bs_debug_unfused_qkv
    f.argtypes = [C.c_void_p, C.c_int]
    f.restype = None
    f(ctx, 1 if on else 0)


def bs_debug_filter_rows(ctx, n_rows):
    """Test hook (not part of the public ABI): per-row threshold of the last filtered accept step:
    (ranking key uint32 as int64, index cut int32, log of the kept mass float32), each [n_rows]."""
    f = lib().bs_debug_copy
    f.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
    f.restype = C.c_int
    key = torch.empty(n_rows, dtype=torch.int32, device="cuda")
    idx = torch.empty(n_rows, dtype=torch.int32, device="cuda")
    lse = torch.empty(n_rows, dtype=torch.float32, device="cuda")
    for which, t in ((7, key), (8, idx), (9, lse)):
        _check(ctx, f(ctx, which, t.data_ptr(), t.numel() * 4, _stream()))
    return key.to(torch.int64) & 0xffffffff, idx, lse
