"""Shared test helpers: glue between the seeded workloads, the oracle and the HIP library.
(Only tests import this; it calls the oracle and the binding side by side.)"""
import numpy as np
import torch

from oracle import accept as OA
from oracle import decoder as OD
from paper_2605_08862_amd import workloads as W

TOL_LOGITS = {W.BS_F32: 1e-4, W.BS_BF16: 2e-2}      # max-abs logit tolerance (spec bar)
NEAR_TIE = 1e-3
FILTER_TIE = 1e-8       # top-p boundary: |cumulative mass - top_p * total| / total below which either set is accepted


def oracle_desc(desc):
    bf16 = desc["dtype"] == W.BS_BF16
    return OD.ModelDesc(desc["n_layers"], desc["d_model"], desc["n_q_heads"], desc["n_kv_heads"], desc["head_dim"],
                        desc["d_ffn"], desc["vocab"], cache_dtype="bf16" if bf16 else "f32",
                        rms_eps=desc["rms_eps"], rope_theta=desc["rope_theta"])


def dev_i32(x, device="cuda:0"):
    return torch.as_tensor(np.ascontiguousarray(x), dtype=torch.int32).to(device)


def dev_f32(x, device="cuda:0"):
    return torch.as_tensor(np.ascontiguousarray(x), dtype=torch.float32).to(device)


def pack_rows(last_token, draft_tokens, draft_len):
    """Token block [last, drafts...] per sequence."""
    return [np.concatenate([[last_token[b]], draft_tokens[b][:draft_len[b]]]).astype(np.int64)
            for b in range(len(draft_len))]


def compare_sampler(gpu, logits_rows, draft_tokens, draft_len, u_accept, u_sample, q_logits_rows=None,
                    temperature=1.0, eos_id=-1, emit_bonus=True, top_k=0, top_p=1.0):
    """Tier A: the oracle's rule on the SAME logits must give the same integers as the device, except
    where the oracle's own margins (or the device's near-tie flags) show a decision within the 1e-3 band.
    Returns (n_exact, n_near_tie, mismatches) and raises on an unexplained mismatch."""
    res = OA.verify_batch(logits_rows, draft_tokens, draft_len, u_accept, u_sample, q_logits_rows, temperature,
                          eos_id, emit_bonus, top_k, top_p)
    row0 = np.concatenate([[0], np.cumsum(np.asarray(draft_len) + 1)])
    n_acc = gpu["n_accepted"].cpu().numpy()
    n_emit = gpu["n_emitted"].cpu().numpy()
    toks = gpu["out_tokens"].cpu().numpy()
    tie = gpu["near_tie"].cpu().numpy().astype(np.uint32)
    exact = near = 0
    for b, r in enumerate(res):
        got = list(toks[b][:n_emit[b]])
        assert all(t == -1 for t in toks[b][n_emit[b]:]), "padding must be -1"
        if n_acc[b] == r.n_accepted and got == [int(t) for t in r.tokens]:
            exact += 1
            continue
        gap_ok = any(g <= NEAR_TIE for g in r.accept_gap)
        samp_ok = r.sample_margin is not None and r.sample_margin <= NEAR_TIE
        if gap_ok or samp_ok or tie[b] != 0:
            near += 1
            continue
        if top_p < 1.0 and temperature > 0 and any(
                OA.kept_tokens(logits_rows[r_], temperature, top_k, top_p)[1] <= FILTER_TIE
                for r_ in range(row0[b], row0[b + 1])):
            near += 1                     # a top-p boundary within rounding of the cumulative mass
            continue
        raise AssertionError("sequence %d: device (%d, %s) vs oracle (%d, %s), no near-tie explains it"
                             % (b, n_acc[b], got, r.n_accepted, r.tokens))
    return exact, near, res


def device_kept(z_row_f32, f_key, f_idx):
    """Indices a device threshold (ranking key, index cut) keeps in a float32 logits row.  The key is the float's
    bit pattern made monotone (sign bit set for non-negative values, all bits inverted for negative ones, -0 == +0):
    token j is kept iff key_j > f_key, or key_j == f_key and j <= f_idx."""
    z = np.ascontiguousarray(z_row_f32, dtype=np.float32) + np.float32(0.0)
    u = z.view(np.uint32).astype(np.int64)
    key = np.where(u & 0x80000000, (~u) & 0xffffffff, u | 0x80000000)
    j = np.arange(z.shape[0])
    return np.flatnonzero((key > int(f_key)) | ((key == int(f_key)) & (j <= int(f_idx))))
