#!/usr/bin/env python3
"""Benchmark of the speculative-verify step on one MI355X.

Workload (configuration "s1p5b_b64_c2048_k8" = benchmark configs[1]): 1.5B-shape bf16 decoder (28 layers,
d=1536, 12 q / 2 kv heads x 128, FFN 8960, vocab 151936, random init), batch 64, context 2048, k = 8 drafts per
sequence, dense proposal q = softmax of a temperature-1 perturbed copy of the target logits (noise scale chosen
for a per-position agreement of 0.7), seeded uniforms.  One step = bs_draft_lookup (on a synthetic pool, through the suffix index
built at set-up; --scan-lookup scans the raw pool instead) +
bs_verify_step + bs_accept_resample + bs_kv_commit, inputs resident in HBM.  All data are synthetic.

Prints ONE JSON line (see the keys below)."""
import argparse
import json
import os
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
MFMA_BF16_PEAK_TFLOPS = 2500.0
AGREEMENT_NOISE = 0.771          # s with 2*Phi(-s/2) = 0.7 (lognormal closed form for E min(p, q))
# HBM bytes per launch of each kernel class at the DEFAULT workload, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (scaled by a plain copy of known size; see profiles/bench_s1p5b_b64_c2048_k8_kernels.txt).  Other workloads: null.
MEASURED_TRAFFIC_BYTES = {"gemm_gate_up": 69.3e6 + 10.3e6, "gemm_down": 48.3e6 + 14.2e6, "attention": 138.3e6 + 1.6e6,
                          "lmhead": 644.3e6 + 23.7e6, "gemm_qkv": 19.7e6 + 2.2e6, "gemm_o": 13.8e6 + 5.2e6}


def build_workload(args):
    dev = "cuda:0"
    desc = W.shape("s1p5b", n_layers=args.layers)
    Bn, ctx, k = args.batch, args.context, args.k
    w = W.make_weights(desc, seed=1002, device=dev)
    eng = Engine(desc, fuse_weights(w, desc["dtype"], dev), Bn, ctx + 2 * k + 2, B_max=Bn, k_max=k)
    # committed context: K, V ~ N(0, (0.02 sqrt(d))^2) rounded to bf16; pages are a permutation of i.i.d. values,
    # so they are filled in place (page encoding of bf16 models: the bf16 value as float16 bits)
    g = torch.Generator(device=dev).manual_seed(2002)
    s = 0.02 * desc["d_model"] ** 0.5
    for l in range(desc["n_layers"]):
        eng.k_pages[l].copy_((torch.randn(eng.k_pages[l].shape, generator=g, device=dev) * s).to(torch.bfloat16).to(torch.float16))
        eng.v_pages[l].copy_((torch.randn(eng.v_pages[l].shape, generator=g, device=dev) * s).to(torch.bfloat16).to(torch.float16))
    eng.ctx_len.fill_(ctx)
    slots = torch.arange(Bn, dtype=torch.int32, device=dev)
    last = torch.randint(0, desc["vocab"], (Bn,), generator=g, device=dev, dtype=torch.int32)
    # drafts and proposal (set-up, untimed): k plain decode steps of the library on the growing prefix
    V = desc["vocab"]
    drafts = torch.zeros(Bn, k, dtype=torch.int32, device=dev)
    q_logits = torch.empty(Bn, k, V, dtype=torch.bfloat16, device=dev)
    zero_len = torch.zeros(Bn, dtype=torch.int32, device=dev)
    one = torch.ones(Bn, dtype=torch.int32, device=dev)
    tok = last.clone()
    for j in range(k):
        z = eng.verify_step(slots, tok, drafts, zero_len, 0, want_logits=True)[:Bn]
        ql = (z + AGREEMENT_NOISE * torch.randn(z.shape, generator=g, device=dev)).to(torch.bfloat16)
        q_logits[:, j] = ql
        tok = torch.multinomial(torch.softmax(ql.float(), dim=-1), 1, generator=g).view(-1).to(torch.int32)
        drafts[:, j] = tok
        eng.kv_commit(slots, one)
    eng.ctx_len.fill_(ctx)                                   # roll the set-up rows back
    ua, us = W.uniforms(3002, Bn, k)
    # synthetic pool for the lookup leg (8 sequences per prompt, 8 rollouts per prompt, median 8k tokens)
    pool = W.make_pool(4002, max(Bn // 8, 1), 8, 8192, V)
    seq_prompt, tails = W.plant_tails(4003, pool, Bn, 8, 4, vocab=V)
    eng.pool_bind(torch.tensor(pool[0]), torch.tensor(pool[1]), torch.tensor(pool[2]))
    index_build_s = None
    if not getattr(args, "scan_lookup", False):                                 # the paper's draft database: a prebuilt suffix index
        t0 = time.perf_counter()
        blob = B.bs_index_build(*pool)                       # host, untimed set-up (once per pool of rollouts)
        index_build_s = time.perf_counter() - t0
        eng.index_bind(blob)
    wl = dict(desc=desc, eng=eng, w=w, slots=slots, last=last, drafts=drafts.contiguous(),
              draft_len=torch.full((Bn,), k, dtype=torch.int32, device=dev),
              q_logits=q_logits.view(Bn * k, V).contiguous(), ua=torch.tensor(ua).to(dev), us=torch.tensor(us).to(dev),
              seq_prompt=torch.tensor(seq_prompt).to(dev), tails=torch.tensor(tails).to(dev),
              ctx0=torch.full((Bn,), ctx, dtype=torch.int32, device=dev), B=Bn, k=k, ctx=ctx,
              index_build_s=index_build_s, pool_tokens=int(len(pool[0])))
    return wl


def one_step(wl):
    eng = wl["eng"]
    eng.ctx_len.copy_(wl["ctx0"])                            # same state every iteration (64 ints)
    eng.draft_lookup(wl["seq_prompt"], wl["tails"], 4, 1, wl["k"])
    eng.verify_step(wl["slots"], wl["last"], wl["drafts"], wl["draft_len"], wl["k"])
    out = eng.accept_resample(wl["drafts"], wl["draft_len"], wl["k"], wl["ua"], wl["us"], q_logits=wl["q_logits"])
    wl["n_commit"] = out["n_accepted"] + 1
    eng.kv_commit(wl["slots"], wl["n_commit"])
    return out


def cpu_baseline(wl, n_seq=8):
    """The oracle, as it stands, on a bounded sample: the first n_seq sequences of the same workload at full depth."""
    from oracle import accept as OA
    from oracle import decoder as OD
    desc, eng, k = wl["desc"], wl["eng"], wl["k"]
    od = OD.ModelDesc(desc["n_layers"], desc["d_model"], desc["n_q_heads"], desc["n_kv_heads"], desc["head_dim"],
                      desc["d_ffn"], desc["vocab"], cache_dtype="bf16", rms_eps=desc["rms_eps"],
                      rope_theta=desc["rope_theta"])
    wn = W.weights_to_numpy(wl["w"])
    last, drafts = wl["last"].cpu().numpy(), wl["drafts"].cpu().numpy()
    ua, us = wl["ua"].cpu().numpy(), wl["us"].cpu().numpy()
    ql = wl["q_logits"].view(wl["B"], k, -1)
    caches = []
    for b in range(n_seq):
        ks, vs = [], []
        for l in range(desc["n_layers"]):
            kk, vv = eng.kv_read(l, b, 0, wl["ctx"])
            ks.append(kk.float().cpu().numpy())
            vs.append(vv.float().cpu().numpy())
        c = OD.SeqCache(od)
        c.fill(ks, vs)
        caches.append(c)
    t0 = time.perf_counter()
    emitted = 0
    for b in range(n_seq):
        z = OD.verify_block(od, wn, caches[b], np.concatenate([[last[b]], drafts[b]]))
        r = OA.verify_sequence(z, drafts[b], ua[b], us[b], ql[b].float().cpu().numpy())
        caches[b].commit(r.n_accepted + 1)
        emitted += len(r.tokens)
    dt = time.perf_counter() - t0
    return dict(value=emitted / dt, unit="tokens/s", cores=torch.get_num_threads(), kind="oracle",
                sample="%d of %d sequences of the same step at full depth (%d layers, context %d, k=%d), %.1f s"
                       % (n_seq, wl["B"], desc["n_layers"], wl["ctx"], k, dt))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--context", type=int, default=2048)
    ap.add_argument("--k", type=int, default=8)
    ap.add_argument("--layers", type=int, default=28)
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
    wl = build_workload(args)
    filtered = args.top_k > 0 or args.top_p < 1.0
    if filtered:
        wl["eng"].set_filter(args.top_k, args.top_p)
    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        out = one_step(wl)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    emitted = accepted = 0
    outs = []
    for _ in range(args.steps):
        outs.append(one_step(wl))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    for o in outs:
        emitted += int(o["n_emitted"].sum().item())
        accepted += int(o["n_accepted"].sum().item())
    fault = wl["eng"].poll_status()
    ms = dt / args.steps * 1e3
    res = {
        "metric": "accepted tokens/s per GPU in verify decode (tokens emitted per second: accepted drafts + the "
                  "recovered/bonus token of each sequence)",
        "value": emitted / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "s1p5b_b%d_c%d_k%d (%s1.5B-shape bf16 decoder, %d layers, dense q, agreement 0.7)"
                               % (args.batch, args.context, args.k,
                                  "BASELINE configs[1]: " if (args.batch, args.context, args.k, args.layers) == (64, 2048, 8, 28)
                                  and not filtered else "NOT the headline configuration: ", args.layers)
                               + (" top_k=%d top_p=%g" % (args.top_k, args.top_p) if filtered else ""),
                   "batch": args.batch, "context": args.context, "k": args.k},
        "accepted_draft_tokens_per_s": accepted / dt,
        "emitted_per_seq_per_step": emitted / (args.steps * args.batch),
        "verify_step_latency_ms": ms,
        "device_fault_word": fault,
        "draft_lookup": {"path": "pool scan" if args.scan_lookup else "prebuilt suffix index",
                         "pool_tokens": wl["pool_tokens"], "index_build_s_host": wl["index_build_s"]},
    }
    res.update(measure_roofline(wl, args))
    if not args.no_cpu_baseline and not filtered:
        res["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(res))


def measure_roofline(wl, args):
    """Per-kernel-class durations measured live with HIP events on the step's own stream (the library's
    bs_profile_* hooks), one pass of `steps` steps per class, after the timed region.  The dominant class is
    reported against its roofline: achieved = ALGORITHMIC bytes (or flops) per launch / mean launch duration."""
    eng, desc = wl["eng"], wl["desc"]
    Bn, k, ctx = wl["B"], wl["k"], wl["ctx"]
    M = Bn * (k + 1)
    d, Hq, Hkv, D, F, V = (desc["d_model"], desc["n_q_heads"], desc["n_kv_heads"], desc["head_dim"], desc["d_ffn"],
                           desc["vocab"])
    kv_bytes_per_token_layer = 2 * Hkv * D * 2                      # K and V rows of one layer, bf16
    algo = {   # class: (bound, units per launch)  units = bytes for hbm, flops for mfma
        "attention": ("hbm", kv_bytes_per_token_layer * Bn * (ctx + k + 1)),
        "gemm_qkv": ("mfma", 2.0 * M * (Hq + 2 * Hkv) * D * d),
        "gemm_o": ("mfma", 2.0 * M * d * Hq * D),
        "gemm_gate_up": ("mfma", 2.0 * M * 2 * F * d),
        "gemm_down": ("mfma", 2.0 * M * d * F),
        "lmhead": ("mfma", 2.0 * M * V * d),
    }
    per_class = {}
    for name, cls in B.PROF_CLASSES.items():
        B.bs_profile_begin(eng.ctx, cls)
        for _ in range(args.steps):
            one_step(wl)
        ms, n = B.bs_profile_end(eng.ctx)
        if n:
            per_class[name] = dict(ms_per_step=ms / args.steps, launches_per_step=n / args.steps,
                                   us_per_launch_events=1e3 * ms / n)
    # An event pair adds a fixed cost to what it brackets; the "empty" class (a pair with nothing in between,
    # once per layer, on the same stream in the same step) measures it, and it is subtracted from every class.
    overhead_us = per_class.pop("empty")["us_per_launch_events"] if "empty" in per_class else 0.0
    for c in per_class.values():
        c["us_per_launch"] = max(c["us_per_launch_events"] - overhead_us, 1e-3)
        c["ms_per_step"] = c["us_per_launch"] * c["launches_per_step"] * 1e-3
    dom = max((c for c in per_class if c in algo), key=lambda c: per_class[c]["ms_per_step"])
    bound, units = algo[dom]
    sec = per_class[dom]["us_per_launch"] * 1e-6
    if bound == "hbm":
        achieved, peak, unit = units / sec / 1e9, HBM_PEAK_GBS, "GB/s"
    else:
        achieved, peak, unit = units / sec / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
    for c, (bnd, u) in algo.items():
        if c in per_class:
            t = per_class[c]["us_per_launch"] * 1e-6
            per_class[c]["bound"] = bnd
            per_class[c]["frac_of_peak"] = (u / t / 1e9 / HBM_PEAK_GBS) if bnd == "hbm" else (u / t / 1e12 / MFMA_BF16_PEAK_TFLOPS)
    default_wl = (args.batch, args.context, args.k, args.layers) == (64, 2048, 8, 28)
    traffic = MEASURED_TRAFFIC_BYTES.get(dom) if default_wl else None
    return {"roofline": {"kernel": dom, "bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                         "frac": achieved / peak, "traffic": traffic,
                         "us_per_launch": per_class[dom]["us_per_launch"],
                         "event_pair_overhead_us": overhead_us},
            "kernel_classes": per_class}


if __name__ == "__main__":
    main()
