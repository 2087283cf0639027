"""GPU check of bs_accept_resample_logits_noalloc, the entry point for callers that cannot allocate: it must return
exactly what bs_accept_resample_logits returns on the same inputs (same kernels, scratch in the library's built-in
device array instead of a workspace), on two calls in a row of which the second is smaller, so that whatever the
first call left in the shared array is seen to do no harm.  The limits are checked on the host."""
import numpy as np
import pytest
import torch

from paper_2605_08862_amd import binding as B
from paper_2605_08862_amd import workloads as W
from paper_2605_08862_amd.runtime import Engine, fuse_weights
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(seed, Bn, k_max, V, q_mode):
    rng = np.random.default_rng(seed)
    k_b = rng.integers(0, k_max + 1, Bn).astype(np.int32)
    M, Td = int(k_b.sum() + Bn), int(k_b.sum())
    logits = rng.normal(0, 2.0, (M, V)).astype(np.float32)
    drafts = rng.integers(0, V, (Bn, k_max)).astype(np.int32)
    r0 = np.concatenate([[0], np.cumsum(k_b + 1)])
    for b in range(Bn):
        for j in range(k_b[b]):
            if rng.random() < 0.6:
                drafts[b, j] = int(np.argmax(logits[r0[b] + j]))
    q = None
    if q_mode and Td > 0:
        q = torch.tensor(rng.normal(0, 2.0, (Td, V)), dtype=torch.bfloat16 if q_mode == "bf16" else torch.float32).to(DEV)
    ua, us = W.uniforms(seed + 1, Bn, k_max)
    return dict(B=Bn, k_max=k_max, V=V, k_b=k_b, logits=H.dev_f32(logits), logits_np=logits, drafts=H.dev_i32(drafts),
                drafts_np=drafts, dl=H.dev_i32(k_b), q=q, ua=H.dev_f32(ua), us=H.dev_f32(us), ua_np=ua, us_np=us)


def _outputs(n, k_max):
    return dict(n_accepted=torch.full((n,), -9, dtype=torch.int32, device=DEV),
                out_tokens=torch.full((n, k_max + 1), -9, dtype=torch.int32, device=DEV),
                n_emitted=torch.full((n,), -9, dtype=torch.int32, device=DEV),
                near_tie=torch.full((n,), -9, dtype=torch.int32, device=DEV))


def _noalloc(x, temperature, eos_id, emit_bonus):
    out = _outputs(x["B"], x["k_max"])
    q_dtype = B.BS_BF16 if (x["q"] is not None and x["q"].dtype == torch.bfloat16) else B.BS_F32
    B.bs_accept_resample_logits_noalloc(x["B"], x["V"], x["logits"], x["drafts"], x["dl"], x["k_max"], x["q"], q_dtype,
                                        float(temperature), eos_id, emit_bonus, x["ua"], x["us"], out["n_accepted"],
                                        out["out_tokens"], out["n_emitted"], out["near_tie"])
    return out


def test_noalloc_equals_the_workspace_entry_point_on_two_calls_in_a_row():
    desc = W.shape("tiny")
    w = W.make_weights(desc, seed=3)
    eng = Engine(desc, fuse_weights(w, desc["dtype"], DEV), 1, 64, B_max=256, k_max=7)
    # first call: 256 sequences x up to 8 rows, vocabulary beyond one statistics tile, dense bf16 proposal;
    # second call: fewer sequences, shorter blocks, smaller vocabulary, one-hot proposal, other options
    cases = [(_inputs(11, 256, 7, 4096, "bf16"), 1.0, -1, True),
             (_inputs(12, 37, 3, 1000, None), 0.7, 5, False),
             (_inputs(13, 5, 0, 50, "f32"), 1.0, -1, True)]
    for x, T, eos, bonus in cases:
        got = _noalloc(x, T, eos, bonus)
        ref = eng.accept_resample(x["drafts"], x["dl"], x["k_max"], x["ua"], x["us"], q_logits=x["q"], temperature=T,
                                  eos_id=eos, emit_bonus=bonus, logits=x["logits"], vocab=x["V"])
        torch.cuda.synchronize()
        for name in ("n_accepted", "out_tokens", "n_emitted", "near_tie"):
            assert torch.equal(got[name].cpu(), ref[name].cpu()), (name, x["B"])
        # and both are the oracle's integers on the same logits
        qn = None if x["q"] is None else x["q"].float().cpu().numpy()
        H.compare_sampler(got, x["logits_np"], x["drafts_np"], x["k_b"], x["ua_np"], x["us_np"], qn, T, eos, bonus)
    assert eng.poll_status() == 0
    eng.close()


def test_noalloc_rejects_sizes_beyond_its_fixed_scratch_and_skips_bad_sequences():
    x = _inputs(21, 4, 3, 64, None)
    x["logits"] = H.dev_f32(np.random.default_rng(22).normal(0, 2.0, (16, 64)))      # room for 4 x (k_max + 1) rows
    out = _outputs(4, 3)
    L = B.lib()
    args = lambda Bn, V, k: (Bn, V, x["logits"].data_ptr(), x["drafts"].data_ptr(), x["dl"].data_ptr(), k, None, 0, 1.0,
                             -1, 1, x["ua"].data_ptr(), x["us"].data_ptr(), out["n_accepted"].data_ptr(),
                             out["out_tokens"].data_ptr(), out["n_emitted"].data_ptr(), out["near_tie"].data_ptr(), None)
    assert L.bs_accept_resample_logits_noalloc(*args(1025, 64, 0)) == B.BS_ESHAPE        # sequences
    assert L.bs_accept_resample_logits_noalloc(*args(512, 64, 4)) == B.BS_ESHAPE         # 2560 packed rows
    assert L.bs_accept_resample_logits_noalloc(*args(4, 262145, 3)) == B.BS_ESHAPE       # vocabulary
    assert L.bs_accept_resample_logits_noalloc(*args(4, 64, 31)) == B.BS_ESHAPE          # k_max
    a = list(args(4, 64, 3)); a[2] = None
    assert L.bs_accept_resample_logits_noalloc(*a) == B.BS_EINVAL
    # a draft length out of range: that sequence is skipped, the others are served
    x["dl"].copy_(H.dev_i32([3, 9, 0, 1]))
    got = _noalloc(x, 1.0, -1, True)
    n_emit = got["n_emitted"].cpu().numpy()
    assert n_emit[1] == 0 and (got["out_tokens"][1].cpu().numpy() == -1).all()
    assert n_emit[0] >= 1 and n_emit[2] == 1 and n_emit[3] >= 1
