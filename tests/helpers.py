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


TIE_SLACK = 1e-4        # float32 evaluation of rho on the device against the oracle's float64


def compare_sampler(gpu, logits_rows, draft_tokens, draft_len, u_accept, u_sample, q_logits_rows=None,
                    temperature=1.0, eos_id=-1, emit_bonus=True, top_k=0, top_p=1.0):
    """Tier A: the oracle's rule on the SAME logits must give the same integers as the device.  A difference is
    excused only by the ORACLE's own margin at the decision where the two part: |rho - u| <= 1e-3 at the first
    accept test they decide differently, or the sampled token's CDF edge within 1e-3 of its mass when the
    accepted prefix agrees (plus, with top-p on, a nucleus boundary within rounding of a cumulative mass).  The
    device's near_tie word is not an excuse but a claim that is checked: every accept test both sides evaluated
    must be flagged iff the oracle finds it inside the band (TIE_SLACK either way), likewise the sampling bit.
    Returns (n_exact, n_near_tie, oracle results) and raises on an unexplained mismatch or a wrong flag."""
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
        same_prefix = n_acc[b] == r.n_accepted
        # accept tests evaluated by both sides: up to and including the first one they may decide differently
        n_common = min(len(r.accept_gap), min(int(n_acc[b]), r.n_accepted) + 1)
        for i in range(n_common):
            flagged = bool(tie[b] >> i & 1)
            gap = r.accept_gap[i]
            assert not (flagged and gap > NEAR_TIE + TIE_SLACK), \
                "sequence %d: device flags accept test %d as a near tie, oracle |rho-u| = %.3g" % (b, i, gap)
            assert not (gap < NEAR_TIE - TIE_SLACK and not flagged), \
                "sequence %d: accept test %d is a near tie (|rho-u| = %.3g) but the device did not flag it" % (b, i, gap)
        if same_prefix and r.sample_margin is not None and temperature > 0 and (got[:-1] == [int(t) for t in r.tokens[:-1]]):
            flagged = bool(tie[b] >> 31 & 1)
            assert not (flagged and r.sample_margin > NEAR_TIE * 1.1), (b, "sampling flag without a near tie", r.sample_margin)
            assert not (r.sample_margin < NEAR_TIE * 0.9 and not flagged), (b, "unflagged sampling near tie", r.sample_margin)
        if same_prefix and got == [int(t) for t in r.tokens]:
            exact += 1
            continue
        if not same_prefix:
            i_div = min(int(n_acc[b]), r.n_accepted)                   # first accept test decided differently
            excused = i_div < len(r.accept_gap) and r.accept_gap[i_div] <= NEAR_TIE
        else:
            excused = r.sample_margin is not None and r.sample_margin <= NEAR_TIE
        if not excused and top_p < 1.0 and temperature > 0 and any(
                OA.kept_tokens(logits_rows[r_], temperature, top_k, top_p)[1] <= FILTER_TIE
                for r_ in range(row0[b], row0[b + 1])):
            excused = True                # a top-p boundary within rounding of the cumulative mass
        if excused:
            near += 1
            continue
        raise AssertionError("sequence %d: device (%d, %s) vs oracle (%d, %s), and the oracle's margin at the "
                             "diverging decision is outside the 1e-3 band" % (b, n_acc[b], got, r.n_accepted, r.tokens))
    return exact, near, res


def tier_c(gpu, oracle_results, seqs):
    """Tier C (end to end): device ids against the oracle's results ON ITS OWN LOGITS for the sequences `seqs`
    (oracle_results[i] belongs to sequence seqs[i]).  Returns (n_same, n_different); differences are legitimate in
    bf16 configurations (the two forwards differ within the logit tolerance and a decision may sit in between),
    which is why they are counted and reported, and each such sequence still has to pass Tier A."""
    n_acc = gpu["n_accepted"].cpu().numpy()
    n_emit = gpu["n_emitted"].cpu().numpy()
    toks = gpu["out_tokens"].cpu().numpy()
    same = 0
    for b, r in zip(seqs, oracle_results):
        same += int(n_acc[b] == r.n_accepted and list(toks[b][:n_emit[b]]) == [int(t) for t in r.tokens])
    return same, len(seqs) - same


def device_kept(z_row_f32, f_key, f_idx):
    """Indices a device threshold (ranking key, index cut) keeps in a float32 logits row.  The key is the float's
    bit pattern made monotone (sign bit set for non-negative values, all bits inverted for negative ones, -0 == +0):
    token j is kept iff key_j > f_key, or key_j == f_key and j <= f_idx."""
    z = np.ascontiguousarray(z_row_f32, dtype=np.float32) + np.float32(0.0)
    u = z.view(np.uint32).astype(np.int64)
    key = np.where(u & 0x80000000, (~u) & 0xffffffff, u | 0x80000000)
    j = np.arange(z.shape[0])
    return np.flatnonzero((key > int(f_key)) | ((key == int(f_key)) & (j <= int(f_idx))))


def oracle_weights_f64(w):
    """float64 copies of the matrices (the embedding stays float32: only single rows of it are read)."""
    wn = W.weights_to_numpy(w)
    c = lambda a: np.asarray(a, dtype=np.float64)
    return {"embed": wn["embed"], "lm_head": c(wn["lm_head"]), "final_norm": c(wn["final_norm"]),
            "layers": [{k: c(v) for k, v in lw.items()} for lw in wn["layers"]]}


def sample_sequences(ctx, k_b, k_max):
    pick = [int(np.argmin(ctx)), int(np.argmax(ctx))]
    zero = np.flatnonzero(k_b == 0)
    full = np.flatnonzero(k_b == k_b.max())
    if len(zero):
        pick.append(int(zero[0]))
    if len(full):
        pick.append(int(full[-1]))
    return sorted(set(pick))


def run_bench_workload_case(name, layers=None):
    """One step of a bench.py workload (optionally cut to `layers` layers) through all three tiers; see
    tests/test_gpu_launch_sizes.py.  Returns (workload, statistics, (drafts, k_b))."""
    import bench
    wl = bench.build_workload(name, layers=layers)
    eng, desc, Bn, k_max = wl["eng"], wl["desc"], wl["B"], wl["k_max"]
    ctx = np.asarray(wl["ctx"])
    eng.ctx_len.copy_(wl["ctx0"])
    if wl["drafts"] is None:                               # configuration 5: drafts straight from the device lookup
        dt, dl = eng.draft_lookup(wl["seq_prompt"], wl["tails"], 4, 1, k_max)
    else:
        dt, dl = wl["drafts"], wl["draft_len"]
    logits = eng.verify_step(wl["slots"], wl["last"], dt, dl, k_max, want_logits=True)
    out = eng.accept_resample(dt, dl, k_max, wl["ua"], wl["us"], q_logits=wl["q_logits"])
    eng.kv_commit(wl["slots"], out["n_accepted"] + 1)
    assert eng.poll_status() == 0
    k_b = dl.cpu().numpy().astype(np.int64)
    drafts = dt.cpu().numpy()
    n_acc, n_emit = out["n_accepted"].cpu().numpy(), out["n_emitted"].cpu().numpy()
    toks = out["out_tokens"].cpu().numpy()
    # ---- properties that hold at any size
    assert eng.ctx_len.cpu().tolist() == [int(c) + int(n) + 1 for c, n in zip(ctx, n_acc)]
    assert eng.kv_lengths(wl["slots"]).cpu().tolist() == eng.ctx_len.cpu().tolist()
    assert ((n_emit == n_acc + 1) & (n_acc >= 0) & (n_acc <= k_b)).all()
    for b in range(Bn):
        assert list(toks[b][:n_acc[b]]) == list(drafts[b][:n_acc[b]])          # accepted prefix is the draft prefix
    M = int(k_b.sum() + Bn)
    row0 = np.concatenate([[0], np.cumsum(k_b + 1)])
    d0 = np.concatenate([[0], np.cumsum(k_b)])
    got = logits[:M].cpu().numpy()
    assert np.isfinite(got).all()
    # ---- Tier A on all sequences
    ua, us = wl["ua"].cpu().numpy(), wl["us"].cpu().numpy()
    ql = None if wl["q_logits"] is None else wl["q_logits"].float().cpu().numpy()
    exact, near, _ = compare_sampler(out, got, drafts, k_b, ua, us, ql)
    assert near <= max(2, 0.03 * Bn), (exact, near)
    # ---- Tier B / C on sampled sequences
    od = oracle_desc(desc)
    wn = oracle_weights_f64(wl["w"])
    last = wl["last"].cpu().numpy()
    picks = sample_sequences(ctx, k_b, k_max)
    worst, oracle_res = 0.0, []
    for b in picks:
        ks, vs = [], []
        for l in range(desc["n_layers"]):
            kk, vv = eng.kv_read(l, b, 0, int(ctx[b]))
            ks.append(kk.float().cpu().numpy())
            vs.append(vv.float().cpu().numpy())
        c = OD.SeqCache(od)
        c.fill(ks, vs)
        k = int(k_b[b])
        ref = OD.verify_block(od, wn, c, np.concatenate([[last[b]], drafts[b][:k]]))
        worst = max(worst, float(np.abs(got[row0[b]:row0[b] + k + 1] - ref).max()))
        oracle_res.append(OA.verify_sequence(ref, drafts[b][:k], ua[b], us[b], None if ql is None else ql[d0[b]:d0[b] + k]))
        # the rows appended by the step (positions c .. c + k), as read back from the pages
        for l in range(desc["n_layers"]):
            kk, vv = eng.kv_read(l, b, int(ctx[b]), k + 1)
            for dev_rows, ref_rows in ((kk, c.k[l][ctx[b]:]), (vv, c.v[l][ctx[b]:])):
                # both sides round to bf16 at rest: values that agree before rounding may land one bf16 step (2^-7
                # relative) apart
                assert (np.abs(dev_rows.float().cpu().numpy() - ref_rows) <= 2e-2 + 2.0 ** -7 * np.abs(ref_rows)).all()
    same, diff = tier_c(out, oracle_res, picks)
    stats = dict(workload=name, rows=M, row_limit=Bn * (k_max + 1), sequences=Bn, sampled=picks,
                 contexts=[int(ctx[b]) for b in picks], k_b=[int(k_b[b]) for b in picks], logits_max_abs=worst,
                 tier_a_exact=exact, tier_a_near_tie=near, tier_c_same=same, tier_c_different=diff,
                 emitted_per_seq=float(n_emit.mean()), drafted_per_seq=float(k_b.mean()))
    print(stats)
    assert worst <= TOL_LOGITS[W.BS_BF16], worst
    return wl, stats, (drafts, k_b)
