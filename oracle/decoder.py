"""Oracle: target-decoder forward for the speculative-verify step (fp64 NumPy).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

The paper treats the target policy as a black box (Sec. 4.1 names Qwen-family
decoders) and only distinguishes "token-wise" operations (linear layers,
normalisation) from the "request-wise" one (attention), Sec. 3.3.  The
architecture below is the pre-norm decoder those models use: RMSNorm, rotary
position encoding with rotate-half pairing, grouped-query causal attention
against a per-sequence KV cache, SwiGLU MLP, untied LM head, no biases.

Verification in one pass over the k+1 positions [last token, draft_1..draft_k]
must equal k+1 plain single-token decode steps (Sec. 2.2: drafts are verified
"in parallel" by the target model).  Both forms are written out separately
here: `decode_token` is the definition, `verify_block` is the one-pass form;
tests require them to agree to fp64 rounding.

Reading taken where the paper is silent: K (after rotary) and V are rounded to
the cache dtype when they are appended (data at rest); nothing else is rounded.

Pin status: invariants only ("parity unpinned" for absolute logit values).
"""
import numpy as np


def round_to_bf16(x):
    """Round fp64 values to the nearest bfloat16 (8 significant bits, ties to
    even) and return them as fp64.  Valid for normal-range magnitudes."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                      # x = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)


def round_for_cache(x, cache_dtype):
    if cache_dtype == "f64":                 # no rounding: used to compare with exact references
        return np.asarray(x, dtype=np.float64)
    if cache_dtype == "bf16":
        return round_to_bf16(x)
    if cache_dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)
    raise ValueError(cache_dtype)


class ModelDesc:
    """Shape and constants of the decoder."""

    def __init__(self, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn,
                 vocab, cache_dtype="f32", rms_eps=1e-6, rope_theta=1e6):
        assert n_q_heads % n_kv_heads == 0 and head_dim % 2 == 0
        self.n_layers, self.d_model = n_layers, d_model
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        self.d_ffn, self.vocab = d_ffn, vocab
        self.cache_dtype, self.rms_eps, self.rope_theta = cache_dtype, rms_eps, rope_theta


class SeqCache:
    """KV cache of ONE sequence: per layer a K and a V array [rows, H_kv, D].

    `length` counts all rows present (committed + tentative).  `committed` is
    the accepted prefix; `commit(n)` keeps n of the tentative rows and drops the
    rest (rollback is simply not keeping them)."""

    def __init__(self, desc):
        self.desc = desc
        shape = (0, desc.n_kv_heads, desc.head_dim)
        self.k = [np.zeros(shape) for _ in range(desc.n_layers)]
        self.v = [np.zeros(shape) for _ in range(desc.n_layers)]
        self.committed = 0

    @property
    def length(self):
        return self.k[0].shape[0]

    def fill(self, k_rows, v_rows):
        """Install committed context directly: lists (per layer) of [c,H_kv,D]."""
        self.k = [np.array(a, dtype=np.float64) for a in k_rows]
        self.v = [np.array(a, dtype=np.float64) for a in v_rows]
        self.committed = self.length

    def append(self, layer, k_new, v_new):
        self.k[layer] = np.concatenate([self.k[layer], k_new], axis=0)
        self.v[layer] = np.concatenate([self.v[layer], v_new], axis=0)

    def commit(self, n_keep):
        tentative = self.length - self.committed
        if not 0 <= n_keep <= tentative:
            raise ValueError("n_keep outside the tentative rows")
        new_len = self.committed + n_keep
        self.k = [a[:new_len] for a in self.k]
        self.v = [a[:new_len] for a in self.v]
        self.committed = new_len


def f64(a):
    return np.asarray(a, dtype=np.float64)


def rmsnorm(x, gain, eps):
    x = f64(x)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * f64(gain)


def rotary(x, pos, theta):
    """Rotate pairs (j, j + D/2) of the last axis by angle pos * theta**(-2j/D)."""
    x = f64(x)
    D = x.shape[-1]
    half = D // 2
    j = np.arange(half, dtype=np.float64)
    ang = float(pos) * theta ** (-2.0 * j / D)
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax(x):
    x = f64(x)
    e = np.exp(x - np.max(x, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def decode_token(desc, w, cache, token):
    """Plain single-token decode: the DEFINITION of the target distribution.

    Appends this token's K/V row to every layer of `cache` (tentatively) and
    returns the logits [V] of the token that follows it."""
    Hq, Hkv, D = desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    G = Hq // Hkv
    pos = cache.length
    h = f64(w["embed"][token]).copy()
    for l in range(desc.n_layers):
        lw = w["layers"][l]
        a = rmsnorm(h, lw["attn_norm"], desc.rms_eps)
        q = (f64(lw["wq"]) @ a).reshape(Hq, D)
        k = (f64(lw["wk"]) @ a).reshape(Hkv, D)
        v = (f64(lw["wv"]) @ a).reshape(Hkv, D)
        q = rotary(q, pos, desc.rope_theta)
        k = rotary(k, pos, desc.rope_theta)
        cache.append(l, round_for_cache(k, desc.cache_dtype)[None],
                     round_for_cache(v, desc.cache_dtype)[None])
        K, V = cache.k[l], cache.v[l]             # [pos+1, Hkv, D]
        o = np.zeros((Hq, D))
        for hq in range(Hq):
            kv = hq // G
            s = K[:, kv, :] @ q[hq] / np.sqrt(D)
            o[hq] = softmax(s) @ V[:, kv, :]
        h = h + f64(lw["wo"]) @ o.reshape(Hq * D)
        m = rmsnorm(h, lw["mlp_norm"], desc.rms_eps)
        h = h + f64(lw["w_down"]) @ (silu(f64(lw["w_gate"]) @ m) * (f64(lw["w_up"]) @ m))
    return f64(w["lm_head"]) @ rmsnorm(h, w["final_norm"], desc.rms_eps)


def verify_block(desc, w, cache, tokens, return_hidden=False):
    """One pass over the n = k+1 positions `tokens` = [last, draft_1..draft_k].

    Row i of the result is the logit vector of the token that follows
    tokens[i] given the cache and tokens[0..i]; draft i+1 is judged by row i.
    Appends n tentative K/V rows per layer."""
    tokens = np.asarray(tokens, dtype=np.int64)
    n = tokens.shape[0]
    Hq, Hkv, D = desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    G = Hq // Hkv
    c = cache.length
    h = f64(np.asarray(w["embed"])[tokens])
    for l in range(desc.n_layers):
        lw = w["layers"][l]
        a = rmsnorm(h, lw["attn_norm"], desc.rms_eps)
        q = (a @ f64(lw["wq"]).T).reshape(n, Hq, D)
        k = (a @ f64(lw["wk"]).T).reshape(n, Hkv, D)
        v = (a @ f64(lw["wv"]).T).reshape(n, Hkv, D)
        for i in range(n):
            q[i] = rotary(q[i], c + i, desc.rope_theta)
            k[i] = rotary(k[i], c + i, desc.rope_theta)
        cache.append(l, round_for_cache(k, desc.cache_dtype),
                     round_for_cache(v, desc.cache_dtype))
        K, V = cache.k[l], cache.v[l]             # [c+n, Hkv, D]
        o = np.zeros((n, Hq, D))
        for hq in range(Hq):
            kv = hq // G
            s = q[:, hq, :] @ K[:, kv, :].T / np.sqrt(D)       # [n, c+n]
            for i in range(n):                                  # causal: row i sees 0..c+i
                o[i, hq] = softmax(s[i, :c + i + 1]) @ V[:c + i + 1, kv, :]
        h = h + o.reshape(n, Hq * D) @ f64(lw["wo"]).T
        m = rmsnorm(h, lw["mlp_norm"], desc.rms_eps)
        h = h + (silu(m @ f64(lw["w_gate"]).T) * (m @ f64(lw["w_up"]).T)) @ f64(lw["w_down"]).T
    hf = rmsnorm(h, w["final_norm"], desc.rms_eps)
    logits = hf @ f64(w["lm_head"]).T
    return (logits, hf) if return_hidden else logits
