"""Seeded synthetic inputs with the shapes of the paper's workloads.

The paper's rollouts use Qwen-family policies on math prompts (Sec. 4.1); neither weights nor
data are available, so every input here is synthetic: random-init decoders of the same shapes,
random token ids, random-filled KV context, seeded uniforms.  This module holds NO arithmetic of
the method (no forward pass, no acceptance rule, no lookup): it only draws numbers.  It serves both
the oracle-side tests and the GPU path."""
import math

import numpy as np
import torch

BS_F32, BS_BF16 = 0, 1

SHAPES = {
    # name: L, d, Hq, Hkv, D, F, V, dtype
    "tiny": dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=1024, vocab=4096, dtype=BS_F32),
    "s1p5b": dict(n_layers=28, d_model=1536, n_q_heads=12, n_kv_heads=2, head_dim=128, d_ffn=8960, vocab=151936, dtype=BS_BF16),
    "s7b": dict(n_layers=28, d_model=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, d_ffn=18944, vocab=152064, dtype=BS_BF16),
    # small bf16 shapes for fast parity tests (same structure: GQA, D=128)
    "mini_bf16": dict(n_layers=2, d_model=256, n_q_heads=6, n_kv_heads=2, head_dim=128, d_ffn=512, vocab=1000, dtype=BS_BF16),
}


def shape(name, **over):
    d = dict(SHAPES[name], rms_eps=1e-6, rope_theta=1e6)
    d.update(over)
    return d


def torch_dtype(desc):
    return torch.float32 if desc["dtype"] == BS_F32 else torch.bfloat16


def make_weights(desc, seed, device="cpu", std=0.02):
    """Random-init weights: matrices and embeddings N(0, std) rounded to the model dtype, norm gains 1.
    Returned per matrix (wq, wk, wv, wo, w_gate, w_up, w_down), row-major [out, in], as torch tensors."""
    g = torch.Generator(device=device).manual_seed(seed)
    td = torch_dtype(desc)
    d, Hq, Hkv, D, F, V = (desc["d_model"], desc["n_q_heads"], desc["n_kv_heads"], desc["head_dim"], desc["d_ffn"],
                           desc["vocab"])

    def mat(r, c):
        return (torch.randn(r, c, generator=g, device=device, dtype=torch.float32) * std).to(td)

    w = {"embed": mat(V, d), "lm_head": mat(V, d), "final_norm": torch.ones(d, device=device), "layers": []}
    for _ in range(desc["n_layers"]):
        w["layers"].append({"attn_norm": torch.ones(d, device=device), "mlp_norm": torch.ones(d, device=device),
                            "wq": mat(Hq * D, d), "wk": mat(Hkv * D, d), "wv": mat(Hkv * D, d), "wo": mat(d, Hq * D),
                            "w_gate": mat(F, d), "w_up": mat(F, d), "w_down": mat(d, F)})
    return w


def weights_to_numpy(w):
    """float32 numpy view of the weights (exact for bf16 values) for the oracle."""
    f = lambda t: t.detach().to("cpu", torch.float32).numpy()
    return {"embed": f(w["embed"]), "lm_head": f(w["lm_head"]), "final_norm": f(w["final_norm"]),
            "layers": [{k: f(v) for k, v in lw.items()} for lw in w["layers"]]}


def context_kv(desc, n_tokens, seed, device="cpu"):
    """Random committed context for one sequence: per layer K, V ~ N(0, (0.02 sqrt(d))^2) in the model dtype,
    the scale a projection of unit-RMS activations by N(0, 0.02) weights would give."""
    g = torch.Generator(device=device).manual_seed(seed)
    td = torch_dtype(desc)
    s = 0.02 * math.sqrt(desc["d_model"])
    shp = (n_tokens, desc["n_kv_heads"], desc["head_dim"])
    return [((torch.randn(shp, generator=g, device=device) * s).to(td), (torch.randn(shp, generator=g, device=device) * s).to(td))
            for _ in range(desc["n_layers"])]


def uniforms(seed, B, k_max):
    """float32 uniforms in [0,1): u_accept [B,k_max], u_sample [B]."""
    rng = np.random.default_rng(seed)
    ua = rng.random((B, max(k_max, 1)), dtype=np.float32)[:, :k_max]
    us = rng.random(B, dtype=np.float32)
    return np.ascontiguousarray(ua), us


def lognormal_lengths(seed, n, median, sigma, lo, hi):
    rng = np.random.default_rng(seed)
    return np.clip(np.exp(rng.normal(math.log(median), sigma, n)), lo, hi).astype(np.int64)


def make_pool(seed, n_prompts, rollouts_per_prompt, median_len, vocab, sigma=1.0, lo=256, hi=32768):
    """Pool of pre-generated rollouts: uniform-random token ids, lognormal lengths.
    Returns (pool_tokens int32, rollout_offsets int64 [R+1], prompt_rollout_begin int32 [P+1])."""
    rng = np.random.default_rng(seed)
    R = n_prompts * rollouts_per_prompt
    lens = lognormal_lengths(seed + 1, R, median_len, sigma, lo, hi)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    toks = rng.integers(0, vocab, size=int(off[-1]), dtype=np.int32)
    prb = (np.arange(n_prompts + 1) * rollouts_per_prompt).astype(np.int32)
    return toks, off, prb


def plant_tails(seed, pool, B, seqs_per_prompt, max_match, p_copy=0.8, p_multi=0.3, vocab=None):
    """Sequence tails for the lookup: with probability p_copy the last max_match tokens are copied from a random
    pool position of the sequence's prompt (so that a suffix match exists); with probability p_multi that span is
    additionally written at two more pool positions of the same prompt so that several continuations compete.
    Mutates pool tokens in place (before they are handed to either implementation).  Returns (seq_prompt, tails)."""
    toks, off, prb = pool
    rng = np.random.default_rng(seed)
    seq_prompt = (np.arange(B) // seqs_per_prompt).astype(np.int32)
    tails = rng.integers(0, vocab, size=(B, max_match), dtype=np.int32)
    for b in range(B):
        if rng.random() >= p_copy:
            continue
        p = seq_prompt[b]
        r = rng.integers(prb[p], prb[p + 1])
        if off[r + 1] - off[r] < max_match + 2:
            continue
        e = rng.integers(off[r] + max_match - 1, off[r + 1] - 1)
        span = toks[e - max_match + 1:e + 1].copy()
        tails[b] = span
        if rng.random() < p_multi:
            for _ in range(2):
                r2 = rng.integers(prb[p], prb[p + 1])
                if off[r2 + 1] - off[r2] < max_match + 2:
                    continue
                e2 = rng.integers(off[r2] + max_match - 1, off[r2 + 1] - 1)
                toks[e2 - max_match + 1:e2 + 1] = span
    return seq_prompt, tails
