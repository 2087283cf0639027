#!/usr/bin/env python3
"""Benchmark of the speculative-verify step on one MI355X.

One step = bs_draft_lookup + bs_verify_step + bs_accept_resample + bs_kv_commit, every input resident in HBM, all
data synthetic (random-init decoders of the named shapes, random committed K/V, seeded uniforms).

Workloads (the benchmark spec `configs`, by index):
  [1] s1p5b_b64_c2048_k8        1.5B shape, batch 64, context 2048, k = 8, dense proposal, agreement 0.7
  [2] s7b_b32_c8192_k8          7B shape, batch 32, context 8192, k = 8, dense proposal, agreement 0.5
  [3] s7b_longtail_b128_k0to16  7B shape, batch 128, contexts clip(lognormal(ln 4096, 1), 512, 32768), k_b ~ U{0..16},
                                dense proposal, per-sequence agreement ~ U(0.2, 0.9)           <- default (headline)
  [4] s1p5b_pool_b256_c16384    1.5B shape, batch 256 = 32 prompts x 8 samples, context 16384, drafts retrieved in the
                                step from a pool of 8 rollouts per prompt (k up to 16), the paper's one-hot proposal
The dense proposal is q_j = softmax(z_j + s eps_j), eps ~ N(0, 1), z_j the target's own logits on the growing draft
prefix (k untimed plain decode steps of the library), s = -2 Phi^-1(a / 2) for agreement a, drafts x_j ~ q_j.

The default run times workload [3] (it carries both the MFMA-bound large-batch GEMMs and the HBM-bound ragged
attention), then adds a `configs` key with a sub-record (ms per step, tokens/s, kernel classes, roofline) for [1],
[2] and [4].  Prints ONE JSON line."""
import argparse
import json
import os
import statistics
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2605_08862_amd import binding as B  # noqa: E402
from paper_2605_08862_amd import workloads as W  # noqa: E402
from paper_2605_08862_amd.runtime import Engine, fuse_weights  # noqa: E402

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0
DTYPE = "f16 MFMA operands, bf16 weights/KV at rest, fp32 accumulate"

CONFIGS = {
    "s1p5b_b64_c2048_k8": dict(index=1, shape="s1p5b", batch=64, context=2048, k=8, agreement=0.7, seed=1002),
    "s7b_b32_c8192_k8": dict(index=2, shape="s7b", batch=32, context=8192, k=8, agreement=0.5, seed=1003),
    "s7b_longtail_b128_k0to16": dict(index=3, shape="s7b", batch=128, context="lognormal", k="ragged", k_max=16,
                                     agreement="uniform", seed=1004),
    "s1p5b_pool_b256_c16384": dict(index=4, shape="s1p5b", batch=256, context=16384, k="lookup", k_max=16,
                                   agreement=None, seed=1005),
}
# not a BASELINE configuration: the batch of the paper's Tab. 1 (128 requests at context 8k, 32 of them with 4 drafts,
# 96 plain decodes) on the 7B shape; used by the parity tests and for the mixed-batch attention comparison
CONFIGS["s7b_tab1_b128_c8192"] = dict(index=-1, shape="s7b", batch=128, context=8192, k="tab1", k_max=4, agreement=0.5,
                                      seed=1006)
DEFAULT = "s7b_longtail_b128_k0to16"
SUB_RECORDS = ["s1p5b_b64_c2048_k8", "s7b_b32_c8192_k8", "s1p5b_pool_b256_c16384"]


def noise_scale(a):
    """s with E min(p, q) = 2 Phi(-s / 2) = a for q = softmax(z + s eps) over a large vocabulary."""
    from scipy.stats import norm
    return float(-2.0 * norm.ppf(a / 2.0))


def check_finite(z, what):
    """Set-up guard: the library's logits go into torch.multinomial, which asserts on the DEVICE (and takes the queue
    down with it) when it is fed a non-finite probability; a non-finite logit ends the program on the host instead."""
    if not bool(torch.isfinite(z).all().item()):
        sys.exit("bench.py: non-finite logits from bs_verify_step at %s; stopping before they reach a sampling op" % what)


def build_workload(name, layers=None, batch=None, scan_lookup=False, all_plain=False):
    cfg = dict(CONFIGS[name])
    dev = "cuda:0"
    desc = W.shape(cfg["shape"], **({"n_layers": layers} if layers else {}))
    Bn = batch or cfg["batch"]
    k_max = cfg.get("k_max", cfg["k"] if isinstance(cfg["k"], int) else 16)
    seed = cfg["seed"]
    rng = np.random.default_rng(seed)
    V = desc["vocab"]
    # ---- per-sequence context length, draft length, agreement
    if cfg["context"] == "lognormal":
        ctx = W.lognormal_lengths(seed + 1, Bn, 4096, 1.0, 512, 32768)
    else:
        ctx = np.full(Bn, cfg["context"], dtype=np.int64)
    if cfg["k"] == "ragged":
        k_b = rng.integers(0, k_max + 1, Bn)
    elif cfg["k"] == "tab1":                                # a quarter of the requests verify 4 drafts, the rest decode
        k_b = np.where(rng.permutation(Bn) < Bn // 4, 4, 0)
    elif cfg["k"] == "lookup":
        k_b = None                                          # set by bs_draft_lookup inside the step
    else:
        k_b = np.full(Bn, cfg["k"], dtype=np.int64)
    if all_plain and k_b is not None:
        k_b = np.zeros(Bn, dtype=np.int64)
    if cfg["agreement"] == "uniform":
        agree = rng.uniform(0.2, 0.9, Bn)
    elif cfg["agreement"] is None:
        agree = None
    else:
        agree = np.full(Bn, cfg["agreement"])
    # ---- model and cache
    w = W.make_weights(desc, seed=seed, device=dev)
    eng = Engine(desc, fuse_weights(w, desc["dtype"], dev), Bn, 0, B_max=Bn, k_max=k_max,
                 slot_tokens=[int(c) + 2 * k_max + 2 for c in ctx])
    # committed context: K, V ~ N(0, (0.02 sqrt(d))^2) rounded to bf16; pages are a permutation of i.i.d. values,
    # so they are filled in place (page encoding of bf16 models: the bf16 value as float16 bits)
    g = torch.Generator(device=dev).manual_seed(seed + 1000)
    s = 0.02 * desc["d_model"] ** 0.5
    for l in range(desc["n_layers"]):
        for pages in (eng.k_pages[l], eng.v_pages[l]):
            step = max(1, (1 << 28) // pages.shape[1])      # at most 1 GiB of float32 temporaries at a time
            for lo in range(0, pages.shape[0], step):
                blk = pages[lo:lo + step]
                blk.copy_((torch.randn(blk.shape, generator=g, device=dev) * s).to(torch.bfloat16).to(torch.float16))
    ctx0 = torch.tensor(ctx, dtype=torch.int32, device=dev)
    eng.ctx_len.copy_(ctx0)
    slots = torch.arange(Bn, dtype=torch.int32, device=dev)
    last = torch.randint(0, V, (Bn,), generator=g, device=dev, dtype=torch.int32)
    wl = dict(name=name, cfg=cfg, desc=desc, eng=eng, w=w, slots=slots, last=last, ctx=ctx, ctx0=ctx0, B=Bn,
              k_max=k_max, q_logits=None, index_build_s=None, pool_tokens=0, lookup_path="none")
    ua, us = W.uniforms(seed + 2000, Bn, k_max)
    wl["ua"], wl["us"] = torch.tensor(ua).to(dev), torch.tensor(us).to(dev)
    # ---- synthetic pool for the lookup leg: 8 rollouts per prompt, lognormal lengths (median 8k), 8 sequences per
    # prompt; tails planted so that 80 % of the sequences have a suffix match
    pool = W.make_pool(seed + 3000, max(Bn // 8, 1), 8, 8192, V)
    seq_prompt, tails = W.plant_tails(seed + 3001, pool, Bn, 8, 4, vocab=V)
    eng.pool_bind(torch.tensor(pool[0]), torch.tensor(pool[1]), torch.tensor(pool[2]))
    wl["lookup_path"] = "pool scan"
    if not scan_lookup:                                     # the paper's draft database: a prebuilt suffix index
        t0 = time.perf_counter()
        blob = B.bs_index_build(*pool)                      # host, untimed set-up (once per pool of rollouts)
        wl["index_build_s"] = time.perf_counter() - t0
        eng.index_bind(blob)
        wl["lookup_path"] = "prebuilt suffix index"
    wl["pool_tokens"] = int(len(pool[0]))
    wl["seq_prompt"], wl["tails"] = torch.tensor(seq_prompt).to(dev), torch.tensor(tails).to(dev)
    wl["pool"], wl["seq_prompt_host"], wl["tails_host"] = pool, seq_prompt, tails
    if k_b is None:
        # drafts come from the lookup inside the step; the step's last token is the tail's newest token
        wl["last"] = wl["tails"][:, -1].clone().contiguous()
        wl["drafts"], wl["draft_len"] = None, None
        wl["k_b"] = None
        return wl
    # ---- drafts and dense proposal (set-up, untimed): k_max plain decode steps of the library on the growing prefix
    sd = torch.tensor([noise_scale(a) for a in agree], dtype=torch.float32, device=dev).view(Bn, 1)
    drafts = torch.zeros(Bn, k_max, dtype=torch.int32, device=dev)
    q_all = torch.empty(Bn, k_max, V, dtype=torch.bfloat16, device=dev)
    zero_len = torch.zeros(Bn, dtype=torch.int32, device=dev)
    one = torch.ones(Bn, dtype=torch.int32, device=dev)
    tok = last.clone()
    for j in range(int(k_b.max())):
        z = eng.verify_step(slots, tok, drafts, zero_len, 0, want_logits=True)[:Bn]
        check_finite(z, "set-up decode step %d of %s" % (j, name))
        ql = (z + sd * torch.randn(z.shape, generator=g, device=dev)).to(torch.bfloat16)
        q_all[:, j] = ql
        tok = torch.multinomial(torch.softmax(ql.float(), dim=-1), 1, generator=g).view(-1).to(torch.int32)
        drafts[:, j] = tok
        eng.kv_commit(slots, one)
    eng.ctx_len.copy_(ctx0)                                  # roll the set-up rows back
    rows = [q_all[b, :int(k_b[b])] for b in range(Bn) if k_b[b] > 0]
    wl["q_logits"] = torch.cat(rows, dim=0).contiguous() if rows else None     # packed [T_d, V], draft-row order
    del q_all
    wl["drafts"] = drafts.contiguous()
    wl["draft_len"] = torch.tensor(k_b, dtype=torch.int32, device=dev)
    wl["k_b"] = k_b
    return wl


def one_step(wl):
    eng = wl["eng"]
    eng.ctx_len.copy_(wl["ctx0"])                            # same state every iteration (B ints)
    dt, dl = eng.draft_lookup(wl["seq_prompt"], wl["tails"], 4, 1, wl["k_max"])
    if wl["drafts"] is not None:                             # configurations with given drafts: the lookup still runs
        dt, dl = wl["drafts"], wl["draft_len"]
    eng.verify_step(wl["slots"], wl["last"], dt, dl, wl["k_max"])
    out = eng.accept_resample(dt, dl, wl["k_max"], wl["ua"], wl["us"], q_logits=wl["q_logits"])
    wl["n_commit"] = out["n_accepted"] + 1
    eng.kv_commit(wl["slots"], wl["n_commit"])
    out["draft_len"] = dl
    return out


def blas_threads():
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 0) for p in threadpool_info() if p.get("user_api") == "blas"]
        return max(n) if n else None
    except Exception:
        return None


def cpu_baseline(wl, n_seq):
    """The oracle, as it stands, on a bounded sample: the first n_seq sequences of the same step at full depth."""
    from oracle import accept as OA
    from oracle import decoder as OD
    import numpy  # noqa: F401  (the oracle's BLAS: its thread count is what `cores` reports)
    desc, eng = wl["desc"], wl["eng"]
    od = OD.ModelDesc(desc["n_layers"], desc["d_model"], desc["n_q_heads"], desc["n_kv_heads"], desc["head_dim"],
                      desc["d_ffn"], desc["vocab"], cache_dtype="bf16", rms_eps=desc["rms_eps"],
                      rope_theta=desc["rope_theta"])
    wn = W.weights_to_numpy(wl["w"])
    last, drafts = wl["last"].cpu().numpy(), wl["drafts"].cpu().numpy()
    k_b = wl["k_b"]
    ua, us = wl["ua"].cpu().numpy(), wl["us"].cpu().numpy()
    d0 = np.concatenate([[0], np.cumsum(k_b)])
    caches = []
    for b in range(n_seq):
        ks, vs = [], []
        for l in range(desc["n_layers"]):
            kk, vv = eng.kv_read(l, b, 0, int(wl["ctx"][b]))
            ks.append(kk.float().cpu().numpy())
            vs.append(vv.float().cpu().numpy())
        c = OD.SeqCache(od)
        c.fill(ks, vs)
        caches.append(c)
    t0 = time.perf_counter()
    emitted = 0
    for b in range(n_seq):
        k = int(k_b[b])
        z = OD.verify_block(od, wn, caches[b], np.concatenate([[last[b]], drafts[b][:k]]))
        ql = wl["q_logits"][d0[b]:d0[b] + k].float().cpu().numpy() if k > 0 else None
        r = OA.verify_sequence(z, drafts[b][:k], ua[b], us[b], ql)
        caches[b].commit(r.n_accepted + 1)
        emitted += len(r.tokens)
    dt = time.perf_counter() - t0
    threads = blas_threads()
    return dict(value=emitted / dt, unit="tokens/s", cores=threads if threads else os.cpu_count(), kind="oracle",
                host_cpus=os.cpu_count(), blas_threads=threads,
                sample="the first %d of %d sequences of the same step at full depth (%d layers; contexts %s, k_b %s), "
                       "%.1f s of oracle time" % (n_seq, wl["B"], desc["n_layers"], [int(c) for c in wl["ctx"][:n_seq]],
                                                  [int(k) for k in k_b[:n_seq]], dt))


def profile_traffic(name):
    """HBM bytes per launch of each kernel class, as the profile step wrote them: the `traffic` lines at the end of
    profiles/<workload>_kernels.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by a plain copy of known size; see
    paper_2605_08862_amd/profile_summary.py).  None when no profile of this workload is there."""
    path = os.path.join(ROOT, "profiles", name + "_kernels.txt")
    out = {}
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "traffic":
                out[f[1]] = float(f[2]) + float(f[3])
    except OSError:
        return None
    return out or None


def profile_clock(name):
    """Shader clock (GHz) and matrix-unit busy share of each kernel class's main kernel, as the counter pass of the
    profile step measured them on a two-layer slice: the `derived` lines of profiles/<workload>_l1_path_counters.txt
    (GRBM_GUI_ACTIVE / 8 / duration, and SQ_VALU_MFMA_BUSY_CYCLES over 1024 SIMDs x cycles).  Context for the
    fraction of the published peak, which assumes 2.4 GHz.  None when no such profile is there."""
    path = os.path.join(ROOT, "profiles", name + "_l1_path_counters.txt")
    out = {}
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "derived":
                out[f[1]] = {"shader_clock_ghz": float(f[2]), "matrix_unit_busy": float(f[3])}
    except OSError:
        return None
    return out or None


def measure(wl, steps, warmup):
    """Times `steps` steps (wall clock around the whole loop, and per step with events on the step's stream)."""
    for _ in range(warmup):
        one_step(wl)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    outs = []
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        outs.append(one_step(wl))
        b.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    emitted = sum(int(o["n_emitted"].sum().item()) for o in outs)
    accepted = sum(int(o["n_accepted"].sum().item()) for o in outs)
    drafted = sum(int(o["draft_len"].sum().item()) for o in outs)
    per_step = [a.elapsed_time(b) for a, b in ev]
    return dict(dt=dt, emitted=emitted, accepted=accepted, drafted=drafted, median_ms=statistics.median(per_step),
                rows=drafted / steps + wl["B"])


def measure_roofline(wl, steps, rows_per_step):
    """Per-kernel-class durations measured live with HIP events on the step's own stream (the library's
    bs_profile_* hooks), one pass of `steps` steps per class, after the timed region.  Every class is priced against
    its roofline: achieved = ALGORITHMIC bytes (or flops) per launch / mean launch duration; the class with the most
    time per step is the `roofline` record."""
    eng, desc = wl["eng"], wl["desc"]
    M = rows_per_step
    d, Hq, Hkv, D, F, V = (desc["d_model"], desc["n_q_heads"], desc["n_kv_heads"], desc["head_dim"], desc["d_ffn"],
                           desc["vocab"])
    kv_bytes_per_token_layer = 2 * Hkv * D * 2                      # K and V rows of one layer, bf16
    tokens = float(np.sum(wl["ctx"])) + M                           # committed context + the step's own rows
    algo = {   # class: (bound, units per launch)  units = bytes for hbm, flops for mfma
        "attention": ("hbm", kv_bytes_per_token_layer * tokens),
        "gemm_qkv": ("mfma", 2.0 * M * (Hq + 2 * Hkv) * D * d),
        "gemm_o": ("mfma", 2.0 * M * d * Hq * D),
        "gemm_gate_up": ("mfma", 2.0 * M * 2 * F * d),
        "gemm_down": ("mfma", 2.0 * M * d * F),
        "lmhead": ("mfma", 2.0 * M * V * d),
    }
    weight_bytes = {"gemm_qkv": 2.0 * (Hq + 2 * Hkv) * D * d, "gemm_o": 2.0 * d * Hq * D, "gemm_gate_up": 4.0 * F * d,
                    "gemm_down": 2.0 * d * F, "lmhead": 2.0 * V * d}
    per_class = {}
    for name, cls in B.PROF_CLASSES.items():
        B.bs_profile_begin(eng.ctx, cls)
        for _ in range(steps):
            one_step(wl)
        ms, n = B.bs_profile_end(eng.ctx)
        if n:
            per_class[name] = dict(ms_per_step=ms / steps, launches_per_step=n / steps,
                                   us_per_launch_events=1e3 * ms / n)
    # An event pair adds a fixed cost to what it brackets; the "empty" class (a pair with nothing in between,
    # once per layer, on the same stream in the same step) measures it, and it is subtracted from every class.
    overhead_us = per_class.pop("empty")["us_per_launch_events"] if "empty" in per_class else 0.0
    for c in per_class.values():
        c["us_per_launch"] = max(c["us_per_launch_events"] - overhead_us, 1e-3)
        c["ms_per_step"] = c["us_per_launch"] * c["launches_per_step"] * 1e-3
    traffic = profile_traffic(wl["name"]) or {}
    clocks = profile_clock(wl["name"]) or {}
    for c, (bnd, u) in algo.items():
        if c not in per_class:
            continue
        t = per_class[c]["us_per_launch"] * 1e-6
        pc = per_class[c]
        # the roofline that bounds the class at this row count: a GEMM below the ridge (2.5 PFLOP/s / 8 TB/s = 312
        # flop per weight byte) is priced against the weight stream
        if bnd == "mfma" and u / weight_bytes[c] < MFMA_F16_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9):
            pc["bound"], pc["algorithmic_units"] = "hbm", weight_bytes[c]
        else:
            pc["bound"], pc["algorithmic_units"] = bnd, u
        if pc["bound"] == "hbm":
            pc["achieved"], pc["peak"], pc["unit"] = pc["algorithmic_units"] / t / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            pc["achieved"], pc["peak"], pc["unit"] = pc["algorithmic_units"] / t / 1e12, MFMA_F16_PEAK_TFLOPS, "TFLOP/s"
        pc["frac_of_peak"] = pc["achieved"] / pc["peak"]
        pc["traffic"] = traffic.get(c)
        if c in clocks:
            pc["profile"] = clocks[c]
    dom = max((c for c in per_class if c in algo), key=lambda c: per_class[c]["ms_per_step"])
    pc = per_class[dom]
    return {"roofline": {"kernel": dom, "bound": pc["bound"], "achieved": pc["achieved"], "peak": pc["peak"],
                         "unit": pc["unit"], "frac": pc["frac_of_peak"], "traffic": pc["traffic"],
                         "profile": pc.get("profile"), "algorithmic_units_per_launch": pc["algorithmic_units"],
                         "us_per_launch": pc["us_per_launch"], "event_pair_overhead_us": overhead_us},
            "kernel_classes": per_class}


def run_config(name, args, steps, warmup, with_cpu, n_cpu_seq=2):
    wl = build_workload(name, layers=args.layers, batch=args.batch, scan_lookup=args.scan_lookup,
                        all_plain=getattr(args, "all_plain", False))
    filtered = args.top_k > 0 or args.top_p < 1.0
    if filtered:
        wl["eng"].set_filter(args.top_k, args.top_p)
    # no device fault during set-up; this poll is also the mark between the set-up steps and the measured phase in a
    # rocprofv3 trace (the status word is cleared by a kernel of its own: see paper_2605_08862_amd/profile_summary.py)
    fault0 = wl["eng"].poll_status()
    if fault0 != 0:
        sys.exit("bench.py: device fault word %d after the set-up of %s" % (fault0, name))
    m = measure(wl, steps, warmup)
    fault = wl["eng"].poll_status()
    cfg = wl["cfg"]
    headline = args.layers is None and args.batch is None and not filtered and not getattr(args, "all_plain", False)
    rec = {
        "value": m["emitted"] / m["dt"], "unit": "tokens/s", "steps": steps, "warmup": warmup,
        "ms_per_step": m["dt"] / steps * 1e3,
        "config": {"workload": "%s (%sBASELINE configs[%d]: %s-shape decoder, %d layers, batch %d)"
                               % (name, "" if headline else "NOT the headline configuration: ", cfg["index"],
                                  cfg["shape"], wl["desc"]["n_layers"], wl["B"])
                               + (" top_k=%d top_p=%g" % (args.top_k, args.top_p) if filtered else ""),
                   "batch": wl["B"], "context_tokens_total": int(np.sum(wl["ctx"])),
                   "context_max": int(np.max(wl["ctx"])), "k_max": wl["k_max"],
                   "rows_per_step": m["rows"], "proposal": "dense bf16 q_logits" if wl["q_logits"] is not None else
                   "one-hot (deterministic drafts from the pool lookup)"},
        "accepted_draft_tokens_per_s": m["accepted"] / m["dt"],
        "emitted_per_seq_per_step": m["emitted"] / (steps * wl["B"]),
        "drafted_per_seq_per_step": m["drafted"] / (steps * wl["B"]),
        "verify_step_latency_ms": m["median_ms"],
        "device_fault_word": fault,
        "draft_lookup": {"path": wl["lookup_path"], "pool_tokens": wl["pool_tokens"],
                         "index_build_s_host": wl["index_build_s"]},
    }
    rec.update(measure_roofline(wl, max(3, steps // 2), m["rows"]))
    if with_cpu and wl["k_b"] is not None and not filtered:
        rec["cpu_baseline"] = cpu_baseline(wl, n_cpu_seq)
    wl["eng"].close()
    del wl
    torch.cuda.empty_cache()
    return rec


def table1_attention(steps=10):
    """The operator-level property of the paper's Tab. 1 (a batch that mixes verification and plain decoding costs the
    attention operator no more than plain decoding): 128 requests at context 8192 on the 7B head configuration, 32 of
    them verifying 4 drafts, against the same batch with no drafts; a two-layer slice (the attention launch does not
    depend on depth).  The paper's figures (0.380 against 0.372 ms, other hardware and kernel) are context only."""
    out = {}
    for key, plain in (("mixed_32x4_drafts_us", False), ("all_plain_us", True)):
        wl = build_workload("s7b_tab1_b128_c8192", layers=2, all_plain=plain)
        for _ in range(3):
            one_step(wl)
        torch.cuda.synchronize()
        B.bs_profile_begin(wl["eng"].ctx, B.PROF_CLASSES["empty"])
        for _ in range(steps):
            one_step(wl)
        ms0, n0 = B.bs_profile_end(wl["eng"].ctx)
        B.bs_profile_begin(wl["eng"].ctx, B.PROF_CLASSES["attention"])
        for _ in range(steps):
            one_step(wl)
        ms, n = B.bs_profile_end(wl["eng"].ctx)
        out[key] = 1e3 * (ms / n - (ms0 / n0 if n0 else 0.0))
        kv_bytes = 2 * wl["desc"]["n_kv_heads"] * wl["desc"]["head_dim"] * 2 * (float(np.sum(wl["ctx"])) + wl["B"])
        out["hbm_frac_" + ("plain" if plain else "mixed")] = kv_bytes / (out[key] * 1e-6) / 1e9 / HBM_PEAK_GBS
        wl["eng"].close()
        del wl
        torch.cuda.empty_cache()
    out["mixed_over_plain"] = out["mixed_32x4_drafts_us"] / out["all_plain_us"]
    out["workload"] = "s7b_tab1_b128_c8192, two-layer slice, attention launch per layer (HIP events, event-pair overhead subtracted)"
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default=DEFAULT, choices=sorted(CONFIGS), help="workload of the main record")
    ap.add_argument("--all-plain", action="store_true",
                    help="every sequence with k_b = 0 (plain decode of the same batch: the comparison of Tab. 1)")
    ap.add_argument("--no-sub", action="store_true", help="skip the sub-records of the other configurations")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size (not the headline then)")
    ap.add_argument("--layers", type=int, default=None, help="override the depth (not the headline then)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--scan-lookup", action="store_true",
                    help="draft lookup by scanning the raw pool instead of walking the prebuilt suffix index")
    ap.add_argument("--top-k", type=int, default=0, help="top-k filter of the target distribution (0: off, the headline)")
    ap.add_argument("--top-p", type=float, default=1.0, help="top-p filter of the target distribution (1.0: off, the headline)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (known traffic) for calibrating rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (sequences shard across GPUs with no collective on the "
                 "step); --gpus %d is not supported" % args.gpus)
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    t_start = time.perf_counter()
    main_rec = run_config(args.config, args, args.steps, args.warmup, not args.no_cpu_baseline)
    res = {
        "metric": "accepted tokens/s per GPU in verify decode (tokens emitted per second: accepted drafts + the "
                  "recovered/bonus token of each sequence)",
        "value": main_rec.pop("value"), "unit": main_rec.pop("unit"), "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_rec.pop("ms_per_step"), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": DTYPE, "data": "synthetic",
    }
    res.update(main_rec)
    if not args.no_sub and args.layers is None and args.batch is None and not args.all_plain:
        subs = {}
        for name in SUB_RECORDS:
            if name == args.config:
                continue
            if time.perf_counter() - t_start > 330:          # keep the whole run well inside ten minutes
                subs[name] = {"skipped": "time budget of the bench run"}
                continue
            try:
                sub_args = argparse.Namespace(**vars(args))
                subs[name] = run_config(name, sub_args, max(5, args.steps // 2), 3, False)
            except (RuntimeError, B.BsError) as e:           # e.g. out of device memory: say so, keep the line
                subs[name] = {"error": str(e)[:300]}
                torch.cuda.empty_cache()
        res["configs"] = subs
        if time.perf_counter() - t_start < 400:
            try:
                res["table1_attention"] = table1_attention()
            except (RuntimeError, B.BsError) as e:
                res["table1_attention"] = {"error": str(e)[:300]}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
