"""Pins for oracle/decoder.py (CPU only).

The decoder has no external reference values (random-init weights), so it is
pinned by (a) an independent forward assembled from torch library routines
(rms_norm, scaled_dot_product_attention with its own causal mask and GQA
handling, silu, linear, rotary as a complex multiplication), (b) the property
that one pass over k+1 positions equals k+1 single-token decodes, (c) textbook
invariants, (d) rollback behaviour of Alg. 1 (the prefix only ever grows by
emitted tokens)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import decoder as D


def make_weights(rng, desc, scale=0.2, gains=True):
    Hq, Hkv, Dh, d, Ff, V = (desc.n_q_heads, desc.n_kv_heads, desc.head_dim,
                             desc.d_model, desc.d_ffn, desc.vocab)
    g = (lambda n: 1.0 + 0.1 * rng.normal(size=n)) if gains else (lambda n: np.ones(n))
    w = {"embed": rng.normal(0, 1.0, (V, d)), "lm_head": rng.normal(0, scale, (V, d)),
         "final_norm": g(d), "layers": []}
    for _ in range(desc.n_layers):
        w["layers"].append({
            "attn_norm": g(d), "mlp_norm": g(d),
            "wq": rng.normal(0, scale, (Hq * Dh, d)), "wk": rng.normal(0, scale, (Hkv * Dh, d)),
            "wv": rng.normal(0, scale, (Hkv * Dh, d)), "wo": rng.normal(0, scale, (d, Hq * Dh)),
            "w_gate": rng.normal(0, scale, (Ff, d)), "w_up": rng.normal(0, scale, (Ff, d)),
            "w_down": rng.normal(0, scale, (d, Ff))})
    return w


def torch_full_forward(desc, w, tokens, origin=0):
    """Whole-sequence causal forward from torch primitives, fp64."""
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    Hq, Hkv, Dh = desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    n = len(tokens)
    h = t(w["embed"])[torch.tensor(tokens)]
    pos = torch.arange(n, dtype=torch.float64) + origin
    inv = desc.rope_theta ** (-torch.arange(0, Dh, 2, dtype=torch.float64) / Dh)
    rot = torch.polar(torch.ones(n, Dh // 2, dtype=torch.float64), pos[:, None] * inv[None])

    def rope(x):                                   # x [n, H, Dh]; pair (j, j+Dh/2) as a complex number
        xc = torch.complex(x[..., :Dh // 2], x[..., Dh // 2:]) * rot[:, None, :]
        return torch.cat([xc.real, xc.imag], dim=-1)

    for lw in w["layers"]:
        a = F.rms_norm(h, (desc.d_model,), t(lw["attn_norm"]), desc.rms_eps)
        q = rope(F.linear(a, t(lw["wq"])).view(n, Hq, Dh)).transpose(0, 1)
        k = rope(F.linear(a, t(lw["wk"])).view(n, Hkv, Dh)).transpose(0, 1)
        v = F.linear(a, t(lw["wv"])).view(n, Hkv, Dh).transpose(0, 1)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True,
                                           enable_gqa=True)[0]
        h = h + F.linear(o.transpose(0, 1).reshape(n, Hq * Dh), t(lw["wo"]))
        m = F.rms_norm(h, (desc.d_model,), t(lw["mlp_norm"]), desc.rms_eps)
        h = h + F.linear(F.silu(F.linear(m, t(lw["w_gate"]))) * F.linear(m, t(lw["w_up"])),
                         t(lw["w_down"]))
    hf = F.rms_norm(h, (desc.d_model,), t(w["final_norm"]), desc.rms_eps)
    return F.linear(hf, t(w["lm_head"])).numpy()


DESC = dict(n_layers=2, d_model=48, n_q_heads=6, n_kv_heads=2, head_dim=8, d_ffn=80, vocab=37)


def test_block_pass_matches_torch_library_forward():
    rng = np.random.default_rng(0)
    desc = D.ModelDesc(**DESC, cache_dtype="f64")
    w = make_weights(rng, desc)
    toks = rng.integers(0, desc.vocab, size=23)
    ref = torch_full_forward(desc, w, toks)
    cache = D.SeqCache(desc)
    got = []
    for lo, hi in [(0, 7), (7, 8), (8, 16), (16, 23)]:       # ragged chunks incl. single token
        got.append(D.verify_block(desc, w, cache, toks[lo:hi]))
        cache.commit(hi - lo)
    np.testing.assert_allclose(np.concatenate(got), ref, rtol=1e-10, atol=1e-11)


def test_block_pass_equals_sequential_decode():
    rng = np.random.default_rng(1)
    desc = D.ModelDesc(**DESC, cache_dtype="bf16")
    w = make_weights(rng, desc)
    toks = rng.integers(0, desc.vocab, size=14)
    c1, c2 = D.SeqCache(desc), D.SeqCache(desc)
    D.verify_block(desc, w, c1, toks[:9]); c1.commit(9)
    for t in toks[:9]:
        D.decode_token(desc, w, c2, t)
    c2.commit(9)
    blk = D.verify_block(desc, w, c1, toks[9:])
    seq = np.stack([D.decode_token(desc, w, c2, t) for t in toks[9:]])
    np.testing.assert_allclose(blk, seq, rtol=1e-11, atol=1e-12)
    for l in range(desc.n_layers):
        np.testing.assert_array_equal(c1.k[l], c2.k[l])
        np.testing.assert_array_equal(c1.v[l], c2.v[l])


def test_rollback_equals_fresh_sequence():
    """verify k drafts -> keep n+1 rows -> next step: same logits as a sequence that only
    ever saw the committed tokens."""
    rng = np.random.default_rng(2)
    desc = D.ModelDesc(**DESC, cache_dtype="bf16")
    w = make_weights(rng, desc)
    prompt = rng.integers(0, desc.vocab, size=6)
    block = rng.integers(0, desc.vocab, size=5)               # last + 4 drafts
    nxt = rng.integers(0, desc.vocab, size=3)
    a = D.SeqCache(desc)
    D.verify_block(desc, w, a, prompt); a.commit(6)
    D.verify_block(desc, w, a, block); a.commit(3)            # 2 drafts accepted (+ last)
    assert a.length == a.committed == 9
    za = D.verify_block(desc, w, a, nxt)
    b = D.SeqCache(desc)
    D.verify_block(desc, w, b, np.concatenate([prompt, block[:3]])); b.commit(9)
    zb = D.verify_block(desc, w, b, nxt)
    np.testing.assert_allclose(za, zb, rtol=1e-11, atol=1e-12)
    with pytest.raises(ValueError):
        a.commit(4)


def test_rotary_is_relative():
    rng = np.random.default_rng(3)
    q, k = rng.normal(size=16), rng.normal(size=16)
    base = D.rotary(q, 5, 1e4) @ D.rotary(k, 2, 1e4)
    np.testing.assert_allclose(D.rotary(q, 1005, 1e4) @ D.rotary(k, 1002, 1e4), base, rtol=1e-9)
    np.testing.assert_allclose(D.rotary(q, 0, 1e4), q)
    # one pair, quarter turn: (x1, x2) -> (-x2, x1)
    np.testing.assert_allclose(D.rotary(np.array([1.0, 2.0]), np.pi / 2, 1e4), [-2.0, 1.0], atol=1e-15)
    desc = D.ModelDesc(**DESC, cache_dtype="f64")
    w = make_weights(rng, desc)
    toks = rng.integers(0, desc.vocab, size=9)
    np.testing.assert_allclose(torch_full_forward(desc, w, toks, origin=300),
                               torch_full_forward(desc, w, toks), rtol=1e-8, atol=1e-9)


def test_gqa_equals_mha_with_repeated_kv_heads():
    rng = np.random.default_rng(4)
    desc = D.ModelDesc(**DESC, cache_dtype="f64")
    w = make_weights(rng, desc)
    G, Dh = desc.n_q_heads // desc.n_kv_heads, desc.head_dim
    mha = D.ModelDesc(**{**DESC, "n_kv_heads": desc.n_q_heads}, cache_dtype="f64")
    w2 = {**w, "layers": []}
    for lw in w["layers"]:
        rep = lambda m: np.repeat(m.reshape(desc.n_kv_heads, Dh, -1), G, axis=0).reshape(-1, m.shape[1])
        w2["layers"].append({**lw, "wk": rep(lw["wk"]), "wv": rep(lw["wv"])})
    toks = rng.integers(0, desc.vocab, size=7)
    np.testing.assert_allclose(D.verify_block(mha, w2, D.SeqCache(mha), toks),
                               D.verify_block(desc, w, D.SeqCache(desc), toks), rtol=1e-11, atol=1e-12)


def test_textbook_special_cases():
    rng = np.random.default_rng(5)
    x = rng.normal(size=(3, 32))
    g = rng.normal(size=32)
    np.testing.assert_allclose(D.rmsnorm(7.5 * x, g, 0.0), D.rmsnorm(x, g, 0.0), rtol=1e-13)
    np.testing.assert_allclose(np.sqrt(np.mean(D.rmsnorm(x, np.ones(32), 0.0) ** 2, axis=-1)), 1.0)
    np.testing.assert_allclose(D.softmax(x + 100.0), D.softmax(x), rtol=1e-12)
    np.testing.assert_allclose(D.silu(x), F.silu(torch.tensor(x)).numpy(), rtol=1e-14)
    # a one-row cache: attention returns that V row, so layer-0 attention output is Wo v
    desc = D.ModelDesc(**{**DESC, "n_layers": 1}, cache_dtype="f64")
    w = make_weights(rng, desc)
    lw = w["layers"][0]
    tok = 11
    cache = D.SeqCache(desc)
    z = D.decode_token(desc, w, cache, tok)
    h0 = w["embed"][tok]
    a = F.rms_norm(torch.tensor(h0), (desc.d_model,), torch.tensor(lw["attn_norm"]), desc.rms_eps).numpy()
    v = lw["wv"] @ a
    G = desc.n_q_heads // desc.n_kv_heads
    o = np.repeat(v.reshape(desc.n_kv_heads, desc.head_dim), G, axis=0).reshape(-1)
    h1 = torch.tensor(h0 + lw["wo"] @ o)
    m = F.rms_norm(h1, (desc.d_model,), torch.tensor(lw["mlp_norm"]), desc.rms_eps)
    h2 = h1 + torch.tensor(lw["w_down"]) @ (F.silu(torch.tensor(lw["w_gate"]) @ m) * (torch.tensor(lw["w_up"]) @ m))
    zz = torch.tensor(w["lm_head"]) @ F.rms_norm(h2, (desc.d_model,), torch.tensor(w["final_norm"]), desc.rms_eps)
    np.testing.assert_allclose(z, zz.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(cache.v[0][0].reshape(-1), v, rtol=1e-13)


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.normal(0, 1, 5000), rng.normal(0, 1e-3, 5000), rng.normal(0, 300, 5000),
                        [1.00390625, 1.01171875, -1.00390625, 0.0]])   # exact ties -> even
    ref = torch.tensor(x, dtype=torch.float64).to(torch.bfloat16).to(torch.float64).numpy()
    got = D.round_to_bf16(x)
    # torch rounds fp64 -> bf16 directly (RNE) on CPU
    np.testing.assert_array_equal(got, ref)
